// Device-wide exclusive prefix sum over int32 (row pointers, compaction offsets, radix-sort digit
// offsets, the row schedule) and over uint64 (cumulative sampling weights).  Large inputs take
// three launches: per-tile sums, a one-block scan of those sums, per-tile scan plus tile offset.
// Small graphs are bound by the number of launches, so up to 1024 tiles every workgroup adds up
// the sums of the tiles before it by itself (two launches), and up to 4 tiles one workgroup
// scans everything (one launch).  Integer arithmetic only, so the result does not depend on
// scheduling.
#include "common.h"

namespace e2eg {

namespace {

constexpr int kThreads = 256;
constexpr int kItems = 8;
constexpr int kTile = kThreads * kItems;
constexpr int kSumThreads = 1024;
constexpr int kScanBatch = 8;

template <typename V>
__device__ __forceinline__ V wave_inclusive_scan(V v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        V t = __shfl_up(v, d, 64);
        if (lane >= d) v += t;
    }
    return v;
}

// Exclusive scan of one value per thread across the block; *total = block sum.
// `lds` holds one value per wavefront.
template <int THREADS, typename V>
__device__ __forceinline__ V block_exclusive_scan(V v, V* total, V* lds) {
    constexpr int kWaves = THREADS / 64;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    V inc = wave_inclusive_scan(v);
    if (lane == 63) lds[wave] = inc;
    __syncthreads();
    V off = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        V s = lds[w];
        if (w < wave) off += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return off + inc - v;
}

// Up to kScanBatch arrays of equal length are scanned by one set of launches: blockIdx.y picks
// the array, and array y keeps its tile sums at sums + y * gridDim.x.
template <typename V>
struct ScanArgs {
    const V* in[kScanBatch];
    V* out[kScanBatch];
    V* total[kScanBatch];
};

template <typename V>
__global__ __launch_bounds__(kThreads) void scan_tile_sums(const ScanArgs<V> a, V* __restrict__ sums,
                                                           int64_t count) {
    __shared__ V lds[kThreads / 64];
    const V* __restrict__ in = a.in[blockIdx.y];
    sums += (int64_t)blockIdx.y * gridDim.x;
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    V s = 0;
#pragma unroll
    for (int k = 0; k < kItems; ++k)
        if (base + k < count) s += in[base + k];
    V total;
    block_exclusive_scan<kThreads, V>(s, &total, lds);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

template <typename V>
__global__ __launch_bounds__(kSumThreads) void scan_sums(const ScanArgs<V> a, V* __restrict__ sums, int64_t nb) {
    __shared__ V lds[kSumThreads / 64];
    V* d_total = a.total[blockIdx.x];
    sums += (int64_t)blockIdx.x * nb;
    V carry = 0;
    for (int64_t base = 0; base < nb; base += kSumThreads) {
        const int64_t i = base + threadIdx.x;
        V v = i < nb ? sums[i] : 0;
        V total;
        V ex = block_exclusive_scan<kSumThreads, V>(v, &total, lds);
        if (i < nb) sums[i] = carry + ex;
        carry += total;
    }
    if (d_total != nullptr && threadIdx.x == 0) *d_total = carry;
}

template <typename V>
__global__ __launch_bounds__(kThreads) void scan_apply(const ScanArgs<V> a, const V* __restrict__ sums,
                                                       int64_t count) {
    __shared__ V lds[kThreads / 64];
    const V* in = a.in[blockIdx.y];
    V* out = a.out[blockIdx.y];
    sums += (int64_t)blockIdx.y * gridDim.x;
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    V v[kItems];
    V s = 0;
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        v[k] = (base + k < count) ? in[base + k] : 0;
        s += v[k];
    }
    V total;
    V ex = block_exclusive_scan<kThreads, V>(s, &total, lds) + sums[blockIdx.x];
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        if (base + k < count) out[base + k] = ex;
        ex += v[k];
    }
}

// The whole input in one workgroup, kSumThreads * kItems values per round.
template <typename V>
__global__ __launch_bounds__(kSumThreads) void scan_one_block(const V* in, V* out, int64_t count,
                                                              V* __restrict__ d_total) {
    __shared__ V lds[kSumThreads / 64];
    V carry = 0;
    for (int64_t base = 0; base < count; base += (int64_t)kSumThreads * kItems) {
        const int64_t at = base + (int64_t)threadIdx.x * kItems;
        V v[kItems];
        V s = 0;
#pragma unroll
        for (int k = 0; k < kItems; ++k) {
            v[k] = (at + k < count) ? in[at + k] : 0;
            s += v[k];
        }
        V total;
        V ex = carry + block_exclusive_scan<kSumThreads, V>(s, &total, lds);
#pragma unroll
        for (int k = 0; k < kItems; ++k) {
            if (at + k < count) out[at + k] = ex;
            ex += v[k];
        }
        carry += total;
    }
    if (d_total != nullptr && threadIdx.x == 0) *d_total = carry;
}

// scan_apply for few tiles: `sums` holds the tiles' own sums, and every workgroup adds up those
// of the tiles before it.
template <typename V>
__global__ __launch_bounds__(kThreads) void scan_apply_few(const ScanArgs<V> a, const V* __restrict__ sums,
                                                           int64_t count) {
    __shared__ V lds[kThreads / 64];
    const V* in = a.in[blockIdx.y];
    V* out = a.out[blockIdx.y];
    V* d_total = a.total[blockIdx.y];
    sums += (int64_t)blockIdx.y * gridDim.x;
    V part = 0;
    for (int64_t i = threadIdx.x; i < (int64_t)blockIdx.x; i += kThreads) part += sums[i];
    V before;
    block_exclusive_scan<kThreads, V>(part, &before, lds);
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    V v[kItems];
    V s = 0;
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        v[k] = (base + k < count) ? in[base + k] : 0;
        s += v[k];
    }
    V total;
    V ex = block_exclusive_scan<kThreads, V>(s, &total, lds) + before;
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        if (base + k < count) out[base + k] = ex;
        ex += v[k];
    }
    if (d_total != nullptr && blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) *d_total = before + total;
}

constexpr int64_t kOneBlockTiles = 4;    // up to here one workgroup scans everything, in one round
constexpr int64_t kFewTiles = 1024;      // up to here the tile offsets are summed in place

// `k` arrays of `count` values each; `ws` holds k * (tiles of one array) values.
template <typename V>
hipError_t exclusive_scan(const ScanArgs<V>& a, int k, int64_t count, void* ws, hipStream_t stream) {
    V* sums = static_cast<V*>(ws);
    const int64_t nb = ceil_div(count > 0 ? count : 0, kTile);
    if (nb <= kOneBlockTiles) {
        for (int y = 0; y < k; ++y)
            scan_one_block<V><<<dim3(1), dim3(kSumThreads), 0, stream>>>(a.in[y], a.out[y], count > 0 ? count : 0,
                                                                         a.total[y]);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)nb, (unsigned)k);
    scan_tile_sums<V><<<grid, dim3(kThreads), 0, stream>>>(a, sums, count);
    if (nb <= kFewTiles) {
        scan_apply_few<V><<<grid, dim3(kThreads), 0, stream>>>(a, sums, count);
        return hipGetLastError();
    }
    scan_sums<V><<<dim3((unsigned)k), dim3(kSumThreads), 0, stream>>>(a, sums, nb);
    scan_apply<V><<<grid, dim3(kThreads), 0, stream>>>(a, sums, count);
    return hipGetLastError();
}

template <typename V>
hipError_t exclusive_scan(const V* in, V* out, int64_t count, V* d_total, void* ws, hipStream_t stream) {
    ScanArgs<V> a = {};
    a.in[0] = in;
    a.out[0] = out;
    a.total[0] = d_total;
    return exclusive_scan<V>(a, 1, count, ws, stream);
}

}  // namespace

size_t scan_workspace_bytes(int64_t count) {
    return align_up((size_t)(ceil_div(count > 0 ? count : 1, kTile)) * sizeof(int32_t));
}

size_t scan_u64_workspace_bytes(int64_t count) {
    return align_up((size_t)(ceil_div(count > 0 ? count : 1, kTile)) * sizeof(uint64_t));
}

hipError_t exclusive_scan_i32(const int32_t* in, int32_t* out, int64_t count, int32_t* d_total,
                              void* ws, hipStream_t stream) {
    return exclusive_scan<int32_t>(in, out, count, d_total, ws, stream);
}

hipError_t exclusive_scan_u64(const uint64_t* in, uint64_t* out, int64_t count, uint64_t* d_total,
                              void* ws, hipStream_t stream) {
    return exclusive_scan<uint64_t>(in, out, count, d_total, ws, stream);
}

hipError_t exclusive_scan_i32_batch(const int32_t* const* in, int32_t* const* out, int k, int64_t count, void* ws,
                                    hipStream_t stream) {
    if (k < 1 || k > kScanBatch) return hipErrorInvalidValue;
    ScanArgs<int32_t> a = {};
    for (int y = 0; y < k; ++y) {
        a.in[y] = in[y];
        a.out[y] = out[y];
        a.total[y] = nullptr;
    }
    return exclusive_scan<int32_t>(a, k, count, ws, stream);
}

}  // namespace e2eg
