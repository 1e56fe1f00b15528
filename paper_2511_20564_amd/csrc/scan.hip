// Device-wide exclusive prefix sum over int32 (row pointers, compaction offsets, radix-sort digit
// offsets, the row schedule) and over uint64 (cumulative sampling weights).  Three launches:
// per-tile sums, a one-block scan of those sums, per-tile scan plus tile offset.  Integer
// arithmetic only, so the result does not depend on scheduling.
#include "common.h"

namespace e2eg {

namespace {

constexpr int kThreads = 256;
constexpr int kItems = 8;
constexpr int kTile = kThreads * kItems;
constexpr int kSumThreads = 1024;

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

template <typename V>
__global__ __launch_bounds__(kThreads) void scan_tile_sums(const V* __restrict__ in, V* __restrict__ sums,
                                                           int64_t count) {
    __shared__ V lds[kThreads / 64];
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
__global__ __launch_bounds__(kSumThreads) void scan_sums(V* __restrict__ sums, int64_t nb, V* __restrict__ d_total) {
    __shared__ V lds[kSumThreads / 64];
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
__global__ __launch_bounds__(kThreads) void scan_apply(const V* in, V* out, const V* __restrict__ sums,
                                                       int64_t count) {
    __shared__ V lds[kThreads / 64];
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

template <typename V>
hipError_t exclusive_scan(const V* in, V* out, int64_t count, V* d_total, void* ws, hipStream_t stream) {
    V* sums = static_cast<V*>(ws);
    const int64_t nb = ceil_div(count > 0 ? count : 0, kTile);
    if (nb > 0) {
        scan_tile_sums<V><<<dim3((unsigned)nb), dim3(kThreads), 0, stream>>>(in, sums, count);
    }
    scan_sums<V><<<dim3(1), dim3(kSumThreads), 0, stream>>>(sums, nb, d_total);
    if (nb > 0) {
        scan_apply<V><<<dim3((unsigned)nb), dim3(kThreads), 0, stream>>>(in, out, sums, count);
    }
    return hipGetLastError();
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

}  // namespace e2eg
