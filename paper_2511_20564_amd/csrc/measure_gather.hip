// Measurement aid, not part of the library: throughput of random 256-byte row gathers on this
// GPU as a function of the table size (L2-resident ... HBM) and of the bytes each lane loads.
// It gives the two rates that bound the neighbour-sum kernel: gathers that hit in L2 and
// gathers that miss.  Stand-alone program: hipcc --offload-arch=gfx950 -O3 measure_gather.hip
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#include <vector>
#include <cstdlib>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)

// Each wave processes `per_wave` indices; row = 256 bytes.  BYTES = bytes per lane per load.
template <int BYTES, int U>
__global__ __launch_bounds__(256) void gather(const char* __restrict__ table, const int* __restrict__ idx,
                                              int per_wave, float* __restrict__ out) {
    constexpr int LANES_PER_ROW = 256 / BYTES;
    constexpr int NB = 64 / LANES_PER_ROW;
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int g = lane / LANES_PER_ROW, c = lane % LANES_PER_ROW;
    const int* my = idx + (size_t)wave * per_wave;
    float acc = 0.f;
    for (int base = 0; base < per_wave; base += 64) {
        int id = my[base + lane];
        for (int t = 0; t < 64; t += U * NB) {
            if (BYTES == 16) {
                uint4 q[U];
#pragma unroll
                for (int u = 0; u < U; ++u) { int j = __shfl(id, t + u * NB + g); q[u] = *reinterpret_cast<const uint4*>(table + (__umul24(j, 256u) + c * 16)); }
#pragma unroll
                for (int u = 0; u < U; ++u) acc += __uint_as_float(q[u].x ^ q[u].y ^ q[u].z ^ q[u].w);
            } else if (BYTES == 8) {
                uint2 q[U];
#pragma unroll
                for (int u = 0; u < U; ++u) { int j = __shfl(id, t + u * NB + g); q[u] = *reinterpret_cast<const uint2*>(table + (__umul24(j, 256u) + c * 8)); }
#pragma unroll
                for (int u = 0; u < U; ++u) acc += __uint_as_float(q[u].x ^ q[u].y);
            } else {
                uint32_t q[U];
#pragma unroll
                for (int u = 0; u < U; ++u) { int j = __shfl(id, t + u * NB + g); q[u] = *reinterpret_cast<const uint32_t*>(table + (__umul24(j, 256u) + c * 4)); }
#pragma unroll
                for (int u = 0; u < U; ++u) acc += __uint_as_float(q[u]);
            }
        }
    }
    if (acc == 123.456f) out[wave] = acc;
}

int main() {
    const int waves = 256 * 32 * 4;      // blocks = waves / 4
    const int per_wave = 1024;
    const size_t total = (size_t)waves * per_wave;
    int* d_idx; float* d_out; char* d_table;
    const size_t max_rows = (size_t)4 << 20;  // 1 GiB table
    CK(hipMalloc(&d_idx, total * 4)); CK(hipMalloc(&d_out, waves * 4)); CK(hipMalloc(&d_table, max_rows * 256));
    CK(hipMemset(d_table, 0, max_rows * 256));
    std::vector<int> h(total);
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    for (size_t rows : {(size_t)2048, (size_t)8192, (size_t)65536, (size_t)524288, max_rows}) {
        uint32_t s = 12345;
        for (size_t i = 0; i < total; ++i) { s = s * 1664525u + 1013904223u; h[i] = (int)((s >> 8) % rows); }
        CK(hipMemcpy(d_idx, h.data(), total * 4, hipMemcpyHostToDevice));
        auto run = [&](const char* name, auto kern) {
            for (int rep = 0; rep < 2; ++rep) {
                CK(hipEventRecord(e0));
                kern<<<waves / 4, 256>>>(d_table, d_idx, per_wave, d_out);
                CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
            }
            float ms; CK(hipEventElapsedTime(&ms, e0, e1));
            printf("table %8.1f MB  %-22s %8.3f ms  %7.2f TB/s gathered\n", rows * 256 / 1e6, name, ms, total * 256.0 / ms / 1e9);
        };
        run("16B/lane x8 in flight", gather<16, 8>);
        run("16B/lane x4 in flight", gather<16, 4>);
        run("8B/lane  x8 in flight", gather<8, 8>);
        run("8B/lane  x16 in flight", gather<8, 16>);
        run("4B/lane  x8 in flight", gather<4, 8>);
        run("4B/lane  x16 in flight", gather<4, 16>);
    }
    return 0;
}
