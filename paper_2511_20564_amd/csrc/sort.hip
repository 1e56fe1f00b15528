// LSD radix sort of 64-bit keys over a chosen bit range, 8-bit digits, stable.  Used to order
// (user, item) pairs for the CSR build and row segments for the schedule.  Integer work only.
#include "common.h"

namespace e2eg {
namespace {

constexpr int kThreads = 256;
constexpr int kSortItems = 8;
constexpr int kSortTile = kThreads * kSortItems;  // keys per block
constexpr int kWaves = kThreads / 64;
constexpr int kFusedBlocks = 128;  // up to this many blocks the scatter adds up its offsets itself

// ---- radix sort, one 8-bit digit per pass --------------------------------------------------
// The table is digit-major [256][nblocks] for the scan, or (BLOCK_MAJOR) [nblocks][256] for a
// scatter that adds up its offsets itself.
template <bool BLOCK_MAJOR>
__global__ __launch_bounds__(kThreads) void sort_histogram(const uint64_t* __restrict__ keys,
                                                           int64_t count, int shift,
                                                           int32_t* __restrict__ hist,
                                                           int32_t nblocks) {
    __shared__ int h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kSortTile;
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
        int64_t idx = base + k * kThreads + threadIdx.x;
        if (idx < count) atomicAdd(&h[(int)((keys[idx] >> shift) & 255)], 1);
    }
    __syncthreads();
    if (BLOCK_MAJOR) hist[(int64_t)blockIdx.x * 256 + threadIdx.x] = h[threadIdx.x];
    else hist[(int64_t)threadIdx.x * nblocks + blockIdx.x] = h[threadIdx.x];
}

// Stable scatter.  A block's tile is split into one contiguous chunk per wavefront; a wavefront
// walks its chunk 64 keys at a time, ranking equal digits by lane order plus a running
// per-wavefront digit count, so ranks follow input order.  The keys are then put in digit order
// inside the tile (in LDS) and written out from there, consecutive threads writing consecutive
// keys: keys of one digit leave as one contiguous run instead of as single 8-byte stores.
// `offs` is the digit-major table [256][nblocks] of scanned offsets, or, with COUNTS, the raw
// block-major histogram [nblocks][256], from which every workgroup then adds up its own 256
// offsets (few blocks: a short loop of coalesced reads that saves the launches of a scan).
template <bool COUNTS>
__global__ __launch_bounds__(kThreads) void sort_scatter(const uint64_t* __restrict__ in,
                                                         uint64_t* __restrict__ out,
                                                         int64_t count, int shift,
                                                         const int32_t* __restrict__ offs,
                                                         int32_t nblocks) {
    __shared__ int wave_cnt[kWaves][256];   // keys of digit d in wavefront w, then their first place in the tile
    __shared__ int wave_tot[kWaves];
    __shared__ int tile_first[256];         // first place of digit d in the tile
    __shared__ int global_first[256];       // where the tile's keys of digit d go
    __shared__ uint64_t tile[kSortTile];
    for (int k = threadIdx.x; k < kWaves * 256; k += kThreads) (&wave_cnt[0][0])[k] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    const int64_t tile_base = (int64_t)blockIdx.x * kSortTile;
    const int64_t chunk = tile_base + (int64_t)wave * (64 * kSortItems);
    uint64_t key[kSortItems];
    int rank[kSortItems];
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        const int64_t idx = chunk + r * 64 + lane;
        const bool valid = idx < count;
        key[r] = valid ? in[idx] : 0ull;
        const int d = (int)((key[r] >> shift) & 255);
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (d >> b) & 1;
            const uint64_t bal = __ballot(valid && bit);
            peers &= bit ? bal : ~bal;
        }
        const int pre = wave_cnt[wave][d];
        const int below = __popcll(peers & lt_mask);
        rank[r] = pre + below;
        if (valid && below == 0) wave_cnt[wave][d] = pre + __popcll(peers);
    }
    __syncthreads();
    {
        // thread d: this tile's keys of digit d (all wavefronts), their first place in the tile
        // (exclusive scan over the digits), and where they go
        const int d = threadIdx.x;
        int mine = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) mine += wave_cnt[w][d];
        int inc = mine;
#pragma unroll
        for (int dlt = 1; dlt < 64; dlt <<= 1) {
            const int t = __shfl_up(inc, dlt, 64);
            if (lane >= dlt) inc += t;
        }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        int first = inc - mine;
#pragma unroll
        for (int w = 0; w < kWaves; ++w)
            if (w < wave) first += wave_tot[w];
        tile_first[d] = first;
        int base;
        if (COUNTS) {
            // keys with a smaller digit anywhere, plus keys with this digit in earlier blocks
            int before = 0, total = 0;
            const int32_t* col = offs + d;
#pragma unroll 16
            for (int b = 0; b < nblocks; ++b) {
                const int c = col[(int64_t)b * 256];
                if (b < (int)blockIdx.x) before += c;
                total += c;
            }
            __syncthreads();   // wave_tot is reused
            int ginc = total;
#pragma unroll
            for (int dlt = 1; dlt < 64; dlt <<= 1) {
                const int t = __shfl_up(ginc, dlt, 64);
                if (lane >= dlt) ginc += t;
            }
            if (lane == 63) wave_tot[wave] = ginc;
            __syncthreads();
            int lower = 0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w)
                if (w < wave) lower += wave_tot[w];
            base = lower + ginc - total + before;
        } else {
            base = offs[(int64_t)d * nblocks + blockIdx.x];
        }
        global_first[d] = base;
        int at = first;   // wave_cnt[w][d] becomes the first tile place of wavefront w's keys of digit d
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const int c = wave_cnt[w][d];
            wave_cnt[w][d] = at;
            at += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        const int64_t idx = chunk + r * 64 + lane;
        if (idx < count) {
            const int d = (int)((key[r] >> shift) & 255);
            tile[wave_cnt[wave][d] + rank[r]] = key[r];
        }
    }
    __syncthreads();
    const int64_t left = count - tile_base;
    const int valid_keys = left < kSortTile ? (int)left : kSortTile;
    for (int p = threadIdx.x; p < valid_keys; p += kThreads) {
        const uint64_t k = tile[p];
        const int d = (int)((k >> shift) & 255);
        out[(int64_t)global_first[d] + (p - tile_first[d])] = k;
    }
}

}  // namespace

size_t radix_sort_workspace_bytes(int64_t count) {
    const int64_t nblocks = ceil_div(count > 0 ? count : 1, kSortTile);
    return align_up((size_t)(256 * nblocks) * sizeof(int32_t)) + scan_workspace_bytes(256 * nblocks);
}

int32_t radix_sort_u64(uint64_t** src, uint64_t** dst, int64_t count, int lo, int nbits, void* ws,
                       hipStream_t stream) {
    if (count <= 0) return E2EG_OK;
    const int32_t nblocks = (int32_t)ceil_div(count, kSortTile);
    int32_t* hist = static_cast<int32_t*>(ws);
    void* scan_ws = static_cast<char*>(ws) + align_up((size_t)(256 * (int64_t)nblocks) * sizeof(int32_t));
    for (int shift = lo; shift < lo + nbits; shift += 8) {
        if (nblocks <= kFusedBlocks) {
            sort_histogram<true><<<dim3(nblocks), dim3(kThreads), 0, stream>>>(*src, count, shift, hist, nblocks);
            E2EG_LAUNCH_CHECK("sort_histogram");
            sort_scatter<true><<<dim3(nblocks), dim3(kThreads), 0, stream>>>(*src, *dst, count, shift, hist, nblocks);
        } else {
            sort_histogram<false><<<dim3(nblocks), dim3(kThreads), 0, stream>>>(*src, count, shift, hist, nblocks);
            E2EG_LAUNCH_CHECK("sort_histogram");
            E2EG_HIP_TRY(exclusive_scan_i32(hist, hist, (int64_t)256 * nblocks, nullptr, scan_ws, stream));
            sort_scatter<false><<<dim3(nblocks), dim3(kThreads), 0, stream>>>(*src, *dst, count, shift, hist, nblocks);
        }
        E2EG_LAUNCH_CHECK("sort_scatter");
        uint64_t* t = *src;
        *src = *dst;
        *dst = t;
    }
    return E2EG_OK;
}

int bits_for(int64_t count) {
    int b = 1;
    while (b < 31 && ((int64_t)1 << b) < count) ++b;
    return b;
}

}  // namespace e2eg
