// Device-wide exclusive prefix sum over int32, used for row pointers, compaction offsets,
// radix-sort digit offsets and the row schedule.  Three launches: per-tile sums, a one-block
// scan of those sums, per-tile scan plus tile offset.  Integer arithmetic only, so the result
// does not depend on scheduling.
#include "common.h"

namespace e2eg {

namespace {

constexpr int kThreads = 256;
constexpr int kItems = 8;
constexpr int kTile = kThreads * kItems;
constexpr int kSumThreads = 1024;

__device__ __forceinline__ int wave_inclusive_scan(int v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int t = __shfl_up(v, d, 64);
        if (lane >= d) v += t;
    }
    return v;
}

// Exclusive scan of one value per thread across the block; *total = block sum.
// `lds` holds one int per wavefront.
template <int THREADS>
__device__ __forceinline__ int block_exclusive_scan(int v, int* total, int* lds) {
    constexpr int kWaves = THREADS / 64;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    int inc = wave_inclusive_scan(v);
    if (lane == 63) lds[wave] = inc;
    __syncthreads();
    int off = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        int s = lds[w];
        if (w < wave) off += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return off + inc - v;
}

__global__ __launch_bounds__(kThreads) void scan_tile_sums(const int32_t* __restrict__ in,
                                                           int32_t* __restrict__ sums,
                                                           int64_t count) {
    __shared__ int lds[kThreads / 64];
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    int s = 0;
#pragma unroll
    for (int k = 0; k < kItems; ++k)
        if (base + k < count) s += in[base + k];
    int total;
    block_exclusive_scan<kThreads>(s, &total, lds);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(kSumThreads) void scan_sums(int32_t* __restrict__ sums, int64_t nb,
                                                         int32_t* __restrict__ d_total) {
    __shared__ int lds[kSumThreads / 64];
    int carry = 0;
    for (int64_t base = 0; base < nb; base += kSumThreads) {
        const int64_t i = base + threadIdx.x;
        int v = i < nb ? sums[i] : 0;
        int total;
        int ex = block_exclusive_scan<kSumThreads>(v, &total, lds);
        if (i < nb) sums[i] = carry + ex;
        carry += total;
    }
    if (d_total != nullptr && threadIdx.x == 0) *d_total = carry;
}

__global__ __launch_bounds__(kThreads) void scan_apply(const int32_t* in, int32_t* out,
                                                       const int32_t* __restrict__ sums,
                                                       int64_t count) {
    __shared__ int lds[kThreads / 64];
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    int v[kItems];
    int s = 0;
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        v[k] = (base + k < count) ? in[base + k] : 0;
        s += v[k];
    }
    int total;
    int ex = block_exclusive_scan<kThreads>(s, &total, lds) + sums[blockIdx.x];
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        if (base + k < count) out[base + k] = ex;
        ex += v[k];
    }
}

}  // namespace

size_t scan_workspace_bytes(int64_t count) {
    return align_up((size_t)(ceil_div(count > 0 ? count : 1, kTile)) * sizeof(int32_t));
}

hipError_t exclusive_scan_i32(const int32_t* in, int32_t* out, int64_t count, int32_t* d_total,
                              void* ws, hipStream_t stream) {
    int32_t* sums = static_cast<int32_t*>(ws);
    const int64_t nb = ceil_div(count > 0 ? count : 0, kTile);
    if (nb > 0) {
        scan_tile_sums<<<dim3((unsigned)nb), dim3(kThreads), 0, stream>>>(in, sums, count);
    }
    scan_sums<<<dim3(1), dim3(kSumThreads), 0, stream>>>(sums, nb, d_total);
    if (nb > 0) {
        scan_apply<<<dim3((unsigned)nb), dim3(kThreads), 0, stream>>>(in, out, sums, count);
    }
    return hipGetLastError();
}

}  // namespace e2eg
