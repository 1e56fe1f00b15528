// e2eg_readout_mean and e2eg_gfae_loss: what the self-supervised branch adds to the propagation.
//   - Layer combination of LightGCN (paper: Section 3.1): the final representation is the mean of
//     all layers, Y = 1/(K+1) (H(0) + H(1) + ... + H(K)).
//   - Graph feature auto-encoder loss with the identity decoder (Section 4.2):
//     L_ssl = ||X - Y||_F^2, whose gradient with respect to Y is 2 (Y - X).
// Both are streaming passes, bound by HBM: readout reads K+1 layers and writes one, the loss reads
// two arrays and (optionally) writes the gradient.  The loss is summed in double, per thread, per
// workgroup in thread order, and over workgroups in index order by a second kernel, so the value
// does not depend on timing.
//
// The mean is a separate pass over stored layers rather than an epilogue of the propagation
// kernel: accumulating it there would need an fp32 running sum read and written once per layer
// (2 * 4 bytes per element and layer) where this pass reads each stored layer once (2 bytes in
// bf16) - fewer bytes, and one rounding of Y.
#include "common.h"

#include <math.h>

namespace e2eg {
namespace {

constexpr int kThreads = 256;
constexpr int kLossBlocks = 16384;  // partial sums of the loss
constexpr int kMaxNormBlocks = 8;   // column blocks (tasks) e2eg_block_norms handles at once
constexpr int kNormBlocks = 4096;   // workgroups of its first pass

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {  // round to nearest even
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

template <bool BF16> struct Chunk;  // 16 bytes of a row as floats
template <> struct Chunk<false> {
    static constexpr int kVec = 4;
    using elem = float;
    static __device__ __forceinline__ void load(const float* p, float (&v)[4]) {
        const float4 q = *reinterpret_cast<const float4*>(p);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    }
    static __device__ __forceinline__ void store(float* p, const float (&v)[4]) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <> struct Chunk<true> {
    static constexpr int kVec = 8;
    using elem = uint16_t;
    static __device__ __forceinline__ void load(const uint16_t* p, float (&v)[8]) {
        const uint4 q = *reinterpret_cast<const uint4*>(p);
        v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
        v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
        v[4] = __uint_as_float(q.z << 16); v[5] = __uint_as_float(q.z & 0xffff0000u);
        v[6] = __uint_as_float(q.w << 16); v[7] = __uint_as_float(q.w & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(uint16_t* p, const float (&v)[8]) {
        *reinterpret_cast<uint4*>(p) = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]),
                                                  pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
    }
};

// Y = (X0 + sum of K layers) / (K + 1), one 16-byte chunk per thread, fp32 arithmetic.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void readout_mean(const typename Chunk<BF16>::elem* __restrict__ x0,
                                                         int64_t ldx,
                                                         const typename Chunk<BF16>::elem* __restrict__ layers,
                                                         int64_t ld, int64_t layer_stride, int32_t K,
                                                         typename Chunk<BF16>::elem* __restrict__ y, int64_t ldy,
                                                         int64_t n, int32_t F) {
    constexpr int V = Chunk<BF16>::kVec;
    const int chunks = F / V;
    const int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (id >= n * chunks) return;
    const int64_t row = id / chunks;
    const int col = (int)(id - row * chunks) * V;
    float acc[V], v[V];
    Chunk<BF16>::load(x0 + row * ldx + col, acc);
    for (int32_t l = 0; l < K; ++l) {
        Chunk<BF16>::load(layers + (int64_t)l * layer_stride + row * ld + col, v);
#pragma unroll
        for (int k = 0; k < V; ++k) acc[k] += v[k];
    }
    const float inv = 1.0f / (float)(K + 1);
#pragma unroll
    for (int k = 0; k < V; ++k) acc[k] *= inv;
    Chunk<BF16>::store(y + row * ldy + col, acc);
}

// Partial sums of sum (x - y)^2 in double (grid-stride over 16-byte chunks), and the gradient
// g = scale2 * (y - x) with scale2 = 2 * grad_scale if g is not null.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void gfae_loss_partial(const typename Chunk<BF16>::elem* __restrict__ x,
                                                              int64_t ldx,
                                                              const typename Chunk<BF16>::elem* __restrict__ y,
                                                              int64_t ldy,
                                                              typename Chunk<BF16>::elem* __restrict__ g,
                                                              int64_t ldg, float scale2, int64_t n, int32_t F,
                                                              double* __restrict__ partial) {
    constexpr int V = Chunk<BF16>::kVec;
    __shared__ double red[kThreads];
    const int chunks = F / V;
    const int64_t total = n * chunks;
    double sum = 0.0;
    for (int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x; id < total; id += (int64_t)gridDim.x * kThreads) {
        const int64_t row = id / chunks;
        const int col = (int)(id - row * chunks) * V;
        float a[V], b[V], d[V];
        Chunk<BF16>::load(x + row * ldx + col, a);
        Chunk<BF16>::load(y + row * ldy + col, b);
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const double e = (double)a[k] - (double)b[k];
            sum += e * e;
            d[k] = scale2 * (b[k] - a[k]);
        }
        if (g) Chunk<BF16>::store(g + row * ldg + col, d);
    }
    red[threadIdx.x] = sum;
    __syncthreads();
    for (int half = kThreads / 2; half > 0; half >>= 1) {   // fixed pairing: the same tree every run
        if ((int)threadIdx.x < half) red[threadIdx.x] += red[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

// One workgroup: thread t adds partials t, t + 256, ... in that order, thread 0 adds the 256 sums.
__global__ __launch_bounds__(kThreads) void gfae_loss_total(const double* __restrict__ partial, int32_t count,
                                                            double* __restrict__ loss) {
    __shared__ double red[kThreads];
    double s = 0.0;
    for (int32_t k = threadIdx.x; k < count; k += kThreads) s += partial[k];
    red[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int k = 0; k < kThreads; ++k) t += red[k];
        *loss = t;
    }
}

// Partial sums of squares of the T column blocks of g ([n][T * F]); block t of workgroup b goes to
// partial[b * T + t].  Grid-stride over 16-byte chunks; a chunk never straddles two blocks because F
// is a multiple of the chunk width.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void block_sumsq_partial(const typename Chunk<BF16>::elem* __restrict__ g,
                                                                int64_t ld, int64_t n, int32_t F, int32_t T,
                                                                double* __restrict__ partial) {
    constexpr int V = Chunk<BF16>::kVec;
    __shared__ double red[kThreads];
    const int chunks_per_block = F / V;
    const int chunks = chunks_per_block * T;
    const int64_t total = n * chunks;
    double sum[kMaxNormBlocks];
#pragma unroll
    for (int t = 0; t < kMaxNormBlocks; ++t) sum[t] = 0.0;
    for (int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x; id < total; id += (int64_t)gridDim.x * kThreads) {
        const int64_t row = id / chunks;
        const int cidx = (int)(id - row * chunks);
        const int t = cidx / chunks_per_block;
        float v[V];
        Chunk<BF16>::load(g + row * ld + (int64_t)cidx * V, v);
        double s = 0.0;
#pragma unroll
        for (int k = 0; k < V; ++k) s += (double)v[k] * (double)v[k];
#pragma unroll
        for (int u = 0; u < kMaxNormBlocks; ++u)
            if (u == t) sum[u] += s;
    }
    for (int t = 0; t < T; ++t) {
        __syncthreads();
        red[threadIdx.x] = sum[t];
        __syncthreads();
        for (int half = kThreads / 2; half > 0; half >>= 1) {   // fixed pairing: the same tree every run
            if ((int)threadIdx.x < half) red[threadIdx.x] += red[threadIdx.x + half];
            __syncthreads();
        }
        if (threadIdx.x == 0) partial[(int64_t)blockIdx.x * T + t] = red[0];
    }
}

// One workgroup per column block t: adds its partials in a fixed order and takes the root.
__global__ __launch_bounds__(kThreads) void block_norms_total(const double* __restrict__ partial, int32_t count,
                                                              int32_t T, double* __restrict__ norms) {
    __shared__ double red[kThreads];
    const int t = blockIdx.x;
    double s = 0.0;
    for (int32_t k = threadIdx.x; k < count; k += kThreads) s += partial[(int64_t)k * T + t];
    red[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double tot = 0.0;
        for (int k = 0; k < kThreads; ++k) tot += red[k];
        norms[t] = sqrt(tot);
    }
}

int32_t check_shape(const char* who, int32_t n, int32_t dtype, int32_t F) {
    if (n < 0) return fail(E2EG_ERR_INVALID_ARG, "%s: negative size", who);
    if (dtype != E2EG_F32 && dtype != E2EG_BF16) return fail(E2EG_ERR_BAD_DTYPE, "%s: dtype %d", who, dtype);
    const int vec = dtype == E2EG_F32 ? 4 : 8;
    if (F <= 0 || F % vec != 0) return fail(E2EG_ERR_INVALID_ARG, "%s: F=%d must be a positive multiple of %d", who, F, vec);
    return E2EG_OK;
}

int32_t check_matrix(const char* who, const char* name, const void* p, int64_t ld, int32_t F, int32_t dtype) {
    const int vec = dtype == E2EG_F32 ? 4 : 8;
    if (!p) return fail(E2EG_ERR_NULL_PTR, "%s: %s is null", who, name);
    if (!aligned_to(p, 16)) return fail(E2EG_ERR_INVALID_ARG, "%s: %s is not 16-byte aligned", who, name);
    if (ld < F || ld % vec != 0)
        return fail(E2EG_ERR_INVALID_ARG, "%s: leading dimension of %s (%lld) must be >= F and a multiple of %d", who,
                    name, (long long)ld, vec);
    return E2EG_OK;
}

}  // namespace
}  // namespace e2eg

using namespace e2eg;

extern "C" int32_t e2eg_readout_mean(int32_t n, int32_t dtype, int32_t F, int32_t K, const void* d_X0, int64_t ldx,
                                     const void* d_layers, int64_t ld, int64_t layer_stride, void* d_Y,
                                     int64_t ldy, void* stream_) {
    const char* who = "readout_mean";
    int32_t st = check_shape(who, n, dtype, F);
    if (st != E2EG_OK) return st;
    if (K < 0) return fail(E2EG_ERR_INVALID_ARG, "%s: K=%d must be >= 0", who, K);
    if ((st = check_matrix(who, "d_X0", d_X0, ldx, F, dtype)) != E2EG_OK) return st;
    if ((st = check_matrix(who, "d_Y", d_Y, ldy, F, dtype)) != E2EG_OK) return st;
    const int vec = dtype == E2EG_F32 ? 4 : 8;
    if (K > 0) {
        if ((st = check_matrix(who, "d_layers", d_layers, ld, F, dtype)) != E2EG_OK) return st;
        if (K > 1 && (layer_stride < (int64_t)n * ld || layer_stride % vec != 0))
            return fail(E2EG_ERR_INVALID_ARG, "%s: layer_stride %lld must be >= n*ld and a multiple of %d", who,
                        (long long)layer_stride, vec);
    }
    if (n == 0) return E2EG_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int64_t total = (int64_t)n * (F / vec);
    const dim3 grid((unsigned)ceil_div(total, kThreads)), blk(kThreads);
    if (dtype == E2EG_F32)
        readout_mean<false><<<grid, blk, 0, stream>>>(static_cast<const float*>(d_X0), ldx,
                                                      static_cast<const float*>(d_layers), ld, layer_stride, K,
                                                      static_cast<float*>(d_Y), ldy, n, F);
    else
        readout_mean<true><<<grid, blk, 0, stream>>>(static_cast<const uint16_t*>(d_X0), ldx,
                                                     static_cast<const uint16_t*>(d_layers), ld, layer_stride, K,
                                                     static_cast<uint16_t*>(d_Y), ldy, n, F);
    E2EG_LAUNCH_CHECK("readout_mean");
    return E2EG_OK;
}

extern "C" size_t e2eg_gfae_loss_workspace_bytes(int32_t n, int32_t F) {
    (void)n;
    (void)F;
    return align_up(sizeof(double) * kLossBlocks);
}

extern "C" int32_t e2eg_gfae_loss(int32_t n, int32_t dtype, int32_t F, const void* d_X, int64_t ldx,
                                  const void* d_Y, int64_t ldy, double* d_loss, void* d_gY, int64_t ldg,
                                  float grad_scale, void* ws, size_t ws_bytes, void* stream_) {
    const char* who = "gfae_loss";
    int32_t st = check_shape(who, n, dtype, F);
    if (st != E2EG_OK) return st;
    if ((st = check_matrix(who, "d_X", d_X, ldx, F, dtype)) != E2EG_OK) return st;
    if ((st = check_matrix(who, "d_Y", d_Y, ldy, F, dtype)) != E2EG_OK) return st;
    if (d_gY && (st = check_matrix(who, "d_gY", d_gY, ldg, F, dtype)) != E2EG_OK) return st;
    if (!d_loss) return fail(E2EG_ERR_NULL_PTR, "%s: d_loss is null", who);
    if (!aligned_to(d_loss, 8)) return fail(E2EG_ERR_INVALID_ARG, "%s: d_loss is not 8-byte aligned", who);
    const size_t need = e2eg_gfae_loss_workspace_bytes(n, F);
    if (!ws || !aligned_to(ws, kAlign) || ws_bytes < need)
        return fail(E2EG_ERR_WORKSPACE, "%s: workspace needs %zu bytes, 256-byte aligned", who, need);
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    double* partial = static_cast<double*>(ws);
    const int vec = dtype == E2EG_F32 ? 4 : 8;
    const int64_t total = (int64_t)n * (F / vec);
    int64_t blocks = ceil_div(total, kThreads);
    if (blocks > kLossBlocks) blocks = kLossBlocks;
    if (blocks < 1) blocks = 1;
    const dim3 grid((unsigned)blocks), blk(kThreads);
    if (dtype == E2EG_F32)
        gfae_loss_partial<false><<<grid, blk, 0, stream>>>(static_cast<const float*>(d_X), ldx,
                                                           static_cast<const float*>(d_Y), ldy,
                                                           static_cast<float*>(d_gY), ldg, 2.0f * grad_scale, n, F,
                                                           partial);
    else
        gfae_loss_partial<true><<<grid, blk, 0, stream>>>(static_cast<const uint16_t*>(d_X), ldx,
                                                          static_cast<const uint16_t*>(d_Y), ldy,
                                                          static_cast<uint16_t*>(d_gY), ldg, 2.0f * grad_scale, n, F,
                                                          partial);
    E2EG_LAUNCH_CHECK("gfae_loss_partial");
    gfae_loss_total<<<dim3(1), dim3(kThreads), 0, stream>>>(partial, (int32_t)blocks, d_loss);
    E2EG_LAUNCH_CHECK("gfae_loss_total");
    return E2EG_OK;
}

extern "C" size_t e2eg_block_norms_workspace_bytes(int32_t n, int32_t F, int32_t T) {
    (void)n;
    (void)F;
    if (T < 1 || T > kMaxNormBlocks) return 0;
    return align_up(sizeof(double) * (size_t)kNormBlocks * (size_t)T);
}

extern "C" int32_t e2eg_block_norms(int32_t n, int32_t dtype, int32_t F, int32_t T, const void* d_G, int64_t ld,
                                    double* d_norms, void* ws, size_t ws_bytes, void* stream_) {
    const char* who = "block_norms";
    int32_t st = check_shape(who, n, dtype, F);
    if (st != E2EG_OK) return st;
    if (T < 1 || T > kMaxNormBlocks) return fail(E2EG_ERR_INVALID_ARG, "%s: T=%d must be in [1, %d]", who, T, kMaxNormBlocks);
    if ((st = check_matrix(who, "d_G", d_G, ld, T * F, dtype)) != E2EG_OK) return st;
    if (!d_norms) return fail(E2EG_ERR_NULL_PTR, "%s: d_norms is null", who);
    if (!aligned_to(d_norms, 8)) return fail(E2EG_ERR_INVALID_ARG, "%s: d_norms is not 8-byte aligned", who);
    const size_t need = e2eg_block_norms_workspace_bytes(n, F, T);
    if (!ws || !aligned_to(ws, kAlign) || ws_bytes < need)
        return fail(E2EG_ERR_WORKSPACE, "%s: workspace needs %zu bytes, 256-byte aligned", who, need);
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    double* partial = static_cast<double*>(ws);
    const int vec = dtype == E2EG_F32 ? 4 : 8;
    const int64_t total = (int64_t)n * (F / vec) * T;
    int64_t blocks = ceil_div(total, kThreads);
    if (blocks > kNormBlocks) blocks = kNormBlocks;
    if (blocks < 1) blocks = 1;
    const dim3 grid((unsigned)blocks), blk(kThreads);
    if (dtype == E2EG_F32)
        block_sumsq_partial<false><<<grid, blk, 0, stream>>>(static_cast<const float*>(d_G), ld, n, F, T, partial);
    else
        block_sumsq_partial<true><<<grid, blk, 0, stream>>>(static_cast<const uint16_t*>(d_G), ld, n, F, T, partial);
    E2EG_LAUNCH_CHECK("block_sumsq_partial");
    block_norms_total<<<dim3((unsigned)T), blk, 0, stream>>>(partial, (int32_t)blocks, T, d_norms);
    E2EG_LAUNCH_CHECK("block_norms_total");
    return E2EG_OK;
}

// Host arithmetic on T scalars per array: no device work.
extern "C" int32_t e2eg_gradnorm_step(int32_t T, const double* h_loss, const double* h_loss0,
                                      const double* h_gnorm, double gamma, double lr, double* h_w,
                                      double* h_meta_loss) {
    const char* who = "gradnorm_step";
    if (T < 1) return fail(E2EG_ERR_INVALID_ARG, "%s: T=%d must be >= 1", who, T);
    if (!h_loss || !h_loss0 || !h_gnorm || !h_w) return fail(E2EG_ERR_NULL_PTR, "%s: null pointer", who);
    double gbar = 0.0, rbar = 0.0;
    for (int32_t i = 0; i < T; ++i) {
        if (!(h_loss0[i] > 0.0) || !(h_w[i] > 0.0))
            return fail(E2EG_ERR_INVALID_ARG, "%s: initial losses and weights must be positive", who);
        gbar += h_w[i] * h_gnorm[i];
        rbar += h_loss[i] / h_loss0[i];
    }
    gbar /= (double)T;
    rbar /= (double)T;
    if (!(rbar > 0.0)) return fail(E2EG_ERR_INVALID_ARG, "%s: the mean loss ratio must be positive", who);
    double meta = 0.0, total = 0.0;
    for (int32_t i = 0; i < T; ++i) {
        const double diff = h_w[i] * h_gnorm[i] - gbar * pow(h_loss[i] / h_loss0[i] / rbar, gamma);
        meta += fabs(diff);
        const double slope = diff > 0.0 ? h_gnorm[i] : (diff < 0.0 ? -h_gnorm[i] : 0.0);
        double w = h_w[i] - lr * slope;
        if (w < 1e-8) w = 1e-8;
        h_w[i] = w;
        total += w;
    }
    for (int32_t i = 0; i < T; ++i) h_w[i] *= (double)T / total;
    if (h_meta_loss) *h_meta_loss = meta;
    return E2EG_OK;
}
