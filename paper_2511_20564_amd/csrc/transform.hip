// e2eg_layer_transform: the dense per-layer update H' = relu(P W) and its backward (paper: the
// update function psi of the generic message-passing layer in Section 3, with the W and sigma of
// the GraphSAGE layer in Section 3.1).
//
// This is the one real contraction on the path, so it runs on the matrix cores: bf16 operands,
// fp32 accumulation, v_mfma_f32_32x32x16_bf16 (wave64; each lane feeds 8 consecutive k of one
// row / column).  The products are computed transposed, D[out column][row], so that a lane ends
// up holding runs of 4 consecutive output columns of ONE row and can store them as 8 bytes.
//   forward : H  = relu(P W)        rows = nodes, k = Fin,  weight tile W^T staged in LDS
//   dP      : dP = dZ W^T           rows = nodes, k = Fout, weight tile W staged in LDS,
//             dZ = gH * [H > 0] formed while loading
//   dW      : dW = P^T dZ           k = nodes: each workgroup reduces a block of nodes into an
//             fp32 partial [Fin][Fout]; partials are added in block order by a second kernel
//             (no atomics, reproducible).
#include "common.h"

#include <mutex>

namespace e2eg {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kRowsPerBlock = 32 * kWaves;   // one 32-row MFMA tile per wavefront
constexpr int kMaxF = 256;
constexpr int kPad = 8;                      // LDS row padding (elements) against bank conflicts
constexpr int kWeightLds = 128 * (128 + kPad);  // elements; also fits 64 x (256 + kPad)
constexpr int kOutLd = 128 + kPad;           // pitch of a wavefront's result rows in LDS (at most 128 columns per workgroup)
constexpr int kTileRows = 64;                // node rows per step of the dW kernel
constexpr int kRowPasses = kTileRows / 32;   // a thread stages one row of every 32
constexpr int kTileLd = kTileRows + 8;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x16 mfma(const uint4 a, const uint4 b, const f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Two floats -> packed bf16, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Keep the bf16 halves of g where the matching half of h is > 0.
__device__ __forceinline__ uint32_t mask_pair(uint32_t g, uint32_t h) {
    uint32_t m = 0;
    if (__uint_as_float(h << 16) > 0.0f) m |= 0x0000ffffu;
    if (__uint_as_float(h & 0xffff0000u) > 0.0f) m |= 0xffff0000u;
    return g & m;
}
__device__ __forceinline__ uint4 mask_vec(uint4 g, uint4 h) {
    return make_uint4(mask_pair(g.x, h.x), mask_pair(g.y, h.y), mask_pair(g.z, h.z), mask_pair(g.w, h.w));
}

// out[r][c] = act( sum_k A[r][k] * B(c, k) ),  A = rows of `a_rows` (masked by `mask_rows` > 0
// when MASKED), B(c, k) = TRANS_W ? w[k][c] : w[c][k].
// grid.x: blocks of `tiles` x 128 rows (the weight tile is staged once per workgroup and serves
// all its row tiles); grid.y: groups of `ngroup` output columns.
// KS: the most k-steps of 16 a row can have (8 for up to 128 input columns).  A wavefront requests
// the rows of its next tile before it multiplies the current one, so that the loads overlap the
// product and the stores.
// EXACT: kdim == 16 * KS and every workgroup has 128 output columns, so that the loops over
// k-steps and column blocks have constant bounds and compile to straight-line code.
template <bool MASKED, bool TRANS_W, bool RELU, int KS, bool EXACT>
__global__ __launch_bounds__(kThreads) void dense_rows(const uint16_t* __restrict__ a_rows,
                                                       const uint16_t* __restrict__ mask_rows,
                                                       const uint16_t* __restrict__ w,
                                                       uint16_t* __restrict__ out, int32_t n,
                                                       int32_t kdim, int32_t ndim, int32_t w_ld,
                                                       int32_t ngroup, int32_t tiles, int32_t stream_out) {
    __shared__ __attribute__((aligned(16))) uint16_t bt[kWeightLds];  // [ngroup][kdim + kPad]
    __shared__ __attribute__((aligned(16))) uint16_t ot[kWaves][16 * kOutLd];  // per wavefront: 16 result rows
    const int ldb = kdim + kPad;
    const int n0 = blockIdx.y * ngroup;
    const int ng = ndim - n0 < ngroup ? ndim - n0 : ngroup;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l32 = lane & 31;
    const int khalf = lane >> 5;
    const int ksteps = EXACT ? KS : kdim / 16;
    const int nblocks = EXACT ? 4 : ng / 32;
    // rows of one tile as this lane feeds them to the matrix core (zeros past the end)
    auto load_rows = [&](int64_t r, uint4 (&va)[KS], uint4 (&vm)[MASKED ? KS : 1]) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            va[ks] = make_uint4(0u, 0u, 0u, 0u);
            if (MASKED) vm[ks] = make_uint4(0u, 0u, 0u, 0u);
            if (ks < ksteps && r < n) {
                const int64_t at = r * kdim + ks * 16 + khalf * 8;
                va[ks] = *reinterpret_cast<const uint4*>(a_rows + at);
                if (MASKED) vm[ks] = *reinterpret_cast<const uint4*>(mask_rows + at);
            }
        }
    };
    const int64_t row_first = (int64_t)blockIdx.x * tiles * kRowsPerBlock + wave * 32 + l32;
    uint4 nxt_a[KS], nxt_m[MASKED ? KS : 1];
    load_rows(row_first, nxt_a, nxt_m);   // in flight while the weight tile is staged
    // stage the weight tile, k contiguous per output column.  Transposing: consecutive lanes take
    // consecutive k, so that their 2-byte LDS writes fall into consecutive banks.
    if (TRANS_W) {
        const int cvecs = ng / 8;
        for (int e = threadIdx.x; e < kdim * cvecs; e += kThreads) {
            const int cv = e / kdim, k = e - cv * kdim;
            const uint4 q = *reinterpret_cast<const uint4*>(w + (int64_t)k * w_ld + n0 + cv * 8);
            const uint32_t words[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bt[(cv * 8 + 2 * j) * ldb + k] = (uint16_t)(words[j] & 0xffffu);
                bt[(cv * 8 + 2 * j + 1) * ldb + k] = (uint16_t)(words[j] >> 16);
            }
        }
    } else {
        const int kvecs = kdim / 8;
        for (int e = threadIdx.x; e < ng * kvecs; e += kThreads) {
            const int c = e / kvecs, kv = e - c * kvecs;
            *reinterpret_cast<uint4*>(bt + c * ldb + kv * 8) =
                *reinterpret_cast<const uint4*>(w + (int64_t)(n0 + c) * w_ld + kv * 8);
        }
    }
    __syncthreads();

#pragma unroll 1
    for (int tile = 0; tile < tiles; ++tile) {
    const int64_t row = row_first + (int64_t)tile * kRowsPerBlock;
    if ((int64_t)row - l32 >= n) return;   // the whole wavefront is past the end

    uint4 areg[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) areg[ks] = MASKED ? mask_vec(nxt_a[ks], nxt_m[ks]) : nxt_a[ks];
    if (tile + 1 < tiles) load_rows(row + kRowsPerBlock, nxt_a, nxt_m);
    f32x16 acc[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[nb][i] = 0.0f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        if (ks < ksteps) {
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                if (nb < nblocks) {
                    const uint4 b = *reinterpret_cast<const uint4*>(bt + (nb * 32 + l32) * ldb + ks * 16 + khalf * 8);
                    acc[nb] = mfma(b, areg[ks], acc[nb]);  // D[out column][row]
                }
            }
        }
    }
    // A lane holds runs of 4 output columns of its row.  Stored from here they would leave as 8-byte
    // pieces, 16 store instructions that each touch 32 rows; instead the wavefront's results go
    // through its LDS tile, 16 rows at a time, and leave as whole rows (a store instruction then
    // writes 4 consecutive rows, 1 KiB in one piece).  Measured at 4 M rows: 634 -> 420 us.
    uint2 pk[4][4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[i] = acc[nb][g4 * 4 + i];
                if (RELU && !(v[i] > 0.0f)) v[i] = 0.0f;
            }
            pk[nb][g4].x = pack_bf16(v[0], v[1]);
            pk[nb][g4].y = pack_bf16(v[2], v[3]);
        }
    }
    uint16_t* ow = ot[wave];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        if ((l32 >> 4) == half) {
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                if (nb < nblocks) {
#pragma unroll
                    for (int g4 = 0; g4 < 4; ++g4)
                        *reinterpret_cast<uint2*>(ow + (l32 & 15) * kOutLd + nb * 32 + g4 * 8 + khalf * 4) = pk[nb][g4];
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int it = 0; it < 4; ++it) {   // 16 rows x 16 chunks of 16 bytes, 64 lanes per pass (128 output columns)
            const int r = it * 4 + (lane >> 4), ch = lane & 15;
            const int64_t grow = row - l32 + half * 16 + r;
            if (grow < n && ch * 8 < ng)
            {
                const uint4 v = *reinterpret_cast<const uint4*>(ow + r * kOutLd + ch * 8);
                if (stream_out) {   // tables far larger than the caches: do not let the results displace the inputs
                    const u32x4 w4 = {v.x, v.y, v.z, v.w};
                    __builtin_nontemporal_store(w4, reinterpret_cast<u32x4*>(out + grow * ndim + n0 + ch * 8));
                } else {
                    *reinterpret_cast<uint4*>(out + grow * ndim + n0 + ch * 8) = v;
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    }
}

// partial[blockIdx.x][c][o] = sum over this block's node rows of P[r][c] * dZ[r][o].
// grid.y / grid.z: groups of 128 columns of P / of dZ.
template <bool MASKED>
__global__ __launch_bounds__(kThreads) void weight_grad_partial(const uint16_t* __restrict__ p,
                                                                const uint16_t* __restrict__ gh,
                                                                const uint16_t* __restrict__ h,
                                                                float* __restrict__ partial, int32_t n,
                                                                int32_t fin, int32_t fout,
                                                                int32_t rows_per_block) {
    __shared__ __attribute__((aligned(16))) uint16_t pt[128 * kTileLd];  // P^T tile  [c][r]
    __shared__ __attribute__((aligned(16))) uint16_t zt[128 * kTileLd];  // dZ^T tile [o][r]
    const int c0 = blockIdx.y * 128, o0 = blockIdx.z * 128;
    const int cg = fin - c0 < 128 ? fin - c0 : 128;
    const int og = fout - o0 < 128 ? fout - o0 : 128;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l32 = lane & 31;
    const int khalf = lane >> 5;
    // staging: consecutive lanes take consecutive tile rows (their 2-byte writes into the
    // transposed tiles then fall into consecutive banks); a thread stages two 8-column chunks
    const int lr = threadIdx.x & 31;   // tile row
    const int cq = threadIdx.x >> 5;   // 8-column chunk cq (and cq + 8)
    const int oblocks = og / 32;
    const bool wave_live = wave * 32 < cg;

    f32x16 acc[4];
#pragma unroll
    for (int ob = 0; ob < 4; ++ob)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[ob][i] = 0.0f;

    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r_end = r_begin + rows_per_block < n ? r_begin + rows_per_block : n;
    // this thread's pieces of one 32-row step: row r0 + lr, column chunks cq and cq + 8 of P and of dZ
    // (dZ with its mask still beside it)
    uint4 qp[2 * kRowPasses], qz[2 * kRowPasses], qh[MASKED ? 2 * kRowPasses : 1];
    auto load_step = [&](int64_t r0) {
#pragma unroll
        for (int half = 0; half < 2 * kRowPasses; ++half) {
            const int cv = cq + (half & 1) * 8;
            const int64_t r = r0 + lr + (half >> 1) * 32;
            qp[half] = make_uint4(0u, 0u, 0u, 0u);
            qz[half] = qp[half];
            if (MASKED) qh[half] = qp[half];
            if (r < r_end) {
                if (cv * 8 < cg) qp[half] = *reinterpret_cast<const uint4*>(p + r * fin + c0 + cv * 8);
                if (cv * 8 < og) {
                    qz[half] = *reinterpret_cast<const uint4*>(gh + r * fout + o0 + cv * 8);
                    if (MASKED) qh[half] = *reinterpret_cast<const uint4*>(h + r * fout + o0 + cv * 8);
                }
            }
        }
    };
    load_step(r_begin);
    for (int64_t r0 = r_begin; r0 < r_end; r0 += kTileRows) {
#pragma unroll
        for (int half = 0; half < 2 * kRowPasses; ++half) {
            const int cv = cq + (half & 1) * 8;
            const int tr = lr + (half >> 1) * 32;   // tile row
            const uint4 z = MASKED ? mask_vec(qz[half], qh[half]) : qz[half];
            const uint32_t wp[4] = {qp[half].x, qp[half].y, qp[half].z, qp[half].w};
            const uint32_t wz[4] = {z.x, z.y, z.z, z.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                pt[(cv * 8 + 2 * j) * kTileLd + tr] = (uint16_t)(wp[j] & 0xffffu);
                pt[(cv * 8 + 2 * j + 1) * kTileLd + tr] = (uint16_t)(wp[j] >> 16);
                zt[(cv * 8 + 2 * j) * kTileLd + tr] = (uint16_t)(wz[j] & 0xffffu);
                zt[(cv * 8 + 2 * j + 1) * kTileLd + tr] = (uint16_t)(wz[j] >> 16);
            }
        }
        __syncthreads();
        if (r0 + kTileRows < r_end) load_step(r0 + kTileRows);   // in flight while this step is multiplied
        if (wave_live) {
#pragma unroll
            for (int ks = 0; ks < kTileRows / 16; ++ks) {
                const uint4 a = *reinterpret_cast<const uint4*>(pt + (wave * 32 + l32) * kTileLd + ks * 16 + khalf * 8);
#pragma unroll
                for (int ob = 0; ob < 4; ++ob) {
                    if (ob < oblocks) {
                        const uint4 b = *reinterpret_cast<const uint4*>(zt + (ob * 32 + l32) * kTileLd + ks * 16 + khalf * 8);
                        acc[ob] = mfma(a, b, acc[ob]);  // D[c][o]
                    }
                }
            }
        }
        __syncthreads();
    }
    if (!wave_live) return;
    float* dst = partial + (int64_t)blockIdx.x * fin * fout;
#pragma unroll
    for (int ob = 0; ob < 4; ++ob) {
        if (ob < oblocks) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int c = c0 + wave * 32 + (i / 4) * 8 + khalf * 4 + (i % 4);
                dst[(int64_t)c * fout + o0 + ob * 32 + l32] = acc[ob][i];
            }
        }
    }
}

// gw[e] = sum over blocks of partial[b][e], in double and in a fixed order: thread (q, j) of a
// workgroup adds blocks q, q + 4, q + 8, ... for element e0 + j; the four sums of an element are
// then added in q order.
constexpr int kReduceElems = 64;   // elements per workgroup
constexpr int kReduceSlices = kThreads / kReduceElems;

__global__ __launch_bounds__(kThreads) void weight_grad_reduce(const float* __restrict__ partial, int32_t nblocks,
                                                               int32_t count, float* __restrict__ gw) {
    __shared__ double red[kReduceSlices][kReduceElems];
    const int j = threadIdx.x % kReduceElems, q = threadIdx.x / kReduceElems;
    const int e = blockIdx.x * kReduceElems + j;
    double s = 0.0;
    if (e < count) {
#pragma unroll 8
        for (int32_t b = q; b < nblocks; b += kReduceSlices) s += (double)partial[(int64_t)b * count + e];
    }
    red[q][j] = s;
    __syncthreads();
    if (q == 0 && e < count) {
        double t = red[0][j];
#pragma unroll
        for (int k = 1; k < kReduceSlices; ++k) t += red[k][j];
        gw[e] = (float)t;
    }
}

// Node rows per workgroup of weight_grad_partial: about one workgroup per compute unit, so that
// few partial matrices are written and read back.
int32_t rows_per_block_for(int32_t n) {
    int64_t r = ceil_div(n > 0 ? n : 1, 256);
    r = (r + kTileRows - 1) / kTileRows * kTileRows;
    return (int32_t)(r < 128 ? 128 : r);
}

template <bool MASKED, bool TRANS_W, bool RELU>
void launch_dense(const void* a, const void* mask, const void* w, void* out, int32_t n, int32_t kdim,
                  int32_t ndim, int32_t w_ld, hipStream_t stream) {
    const int32_t ngroup = kdim > 128 ? 64 : 128;
    int64_t tiles = ceil_div(n, (int64_t)kRowsPerBlock * 512);   // keep at least ~512 workgroups
    tiles = tiles < 1 ? 1 : (tiles > 8 ? 8 : tiles);
    const dim3 grid((unsigned)ceil_div(n, kRowsPerBlock * tiles), (unsigned)ceil_div(ndim, ngroup));
    // streaming stores once the result is far larger than the caches (measured: 5 % at 4 M rows); below
    // that the next kernel of a mini-batch step finds the rows in the caches if they are written normally
    const int32_t stream_out = (int64_t)n * ndim * 2 > (64ll << 20) ? 1 : 0;
    if (kdim == 128 && ndim % 128 == 0)
        dense_rows<MASKED, TRANS_W, RELU, 8, true><<<grid, dim3(kThreads), 0, stream>>>(
            static_cast<const uint16_t*>(a), static_cast<const uint16_t*>(mask), static_cast<const uint16_t*>(w),
            static_cast<uint16_t*>(out), n, kdim, ndim, w_ld, ngroup, (int32_t)tiles, stream_out);
    else if (kdim <= 128)
        dense_rows<MASKED, TRANS_W, RELU, 8, false><<<grid, dim3(kThreads), 0, stream>>>(
            static_cast<const uint16_t*>(a), static_cast<const uint16_t*>(mask), static_cast<const uint16_t*>(w),
            static_cast<uint16_t*>(out), n, kdim, ndim, w_ld, ngroup, (int32_t)tiles, stream_out);
    else
        dense_rows<MASKED, TRANS_W, RELU, kMaxF / 16, false><<<grid, dim3(kThreads), 0, stream>>>(
            static_cast<const uint16_t*>(a), static_cast<const uint16_t*>(mask), static_cast<const uint16_t*>(w),
            static_cast<uint16_t*>(out), n, kdim, ndim, w_ld, ngroup, (int32_t)tiles, stream_out);
}

}  // namespace
}  // namespace e2eg

using namespace e2eg;

extern "C" size_t e2eg_layer_transform_workspace_bytes(int32_t mode, int32_t n, int32_t Fin,
                                                       int32_t Fout, int32_t dtype) {
    if (n < 0 || Fin <= 0 || Fout <= 0 || dtype != E2EG_BF16) return 0;
    if (mode != E2EG_TRANSFORM_BWD) return kAlign;
    const int64_t blocks = ceil_div(n > 0 ? n : 1, rows_per_block_for(n));
    return align_up((size_t)blocks * (size_t)Fin * (size_t)Fout * sizeof(float));
}

// ---- the same call for callers that cannot allocate ------------------------------------------
// The partial weight-gradient matrices live in a device array that is part of the library's code
// object, so no workspace has to come from anywhere.  Each GPU holds its own copy of the array at
// its own address; host code never uses the array's name as an address, only the pointer
// hipGetSymbolAddress returns for the current device, looked up once per device and kept.
static __device__ __align__(256) float scratch[E2EG_TRANSFORM_STATIC_SCRATCH_BYTES / sizeof(float)];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices];   // address of `scratch` on each device, null until looked up

int32_t static_scratch_of_current_device(float** out) {
    int dev = -1;
    E2EG_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(E2EG_ERR_HIP, "layer_transform_noalloc: device index %d", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        float* p = nullptr;
        E2EG_HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)));
        if (!p) return fail(E2EG_ERR_HIP, "layer_transform_noalloc: the scratch array has no address on device %d", dev);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return E2EG_OK;
}
}  // namespace

namespace {
// Shared by the two entry points: `ws` is the caller's workspace, or the library's static scratch
// array (static_scratch: looked up here once the arguments have passed; a need beyond its size is a
// CAPACITY error).
int32_t transform_impl(const char* who, bool static_scratch, int32_t mode, int32_t n, int32_t Fin, int32_t Fout,
                       int32_t dtype, int32_t relu, const void* d_P, const void* d_W, void* d_H, const void* d_gH,
                       void* d_gP, float* d_gW, void* ws, size_t ws_bytes, void* stream_) {
    if (mode != E2EG_TRANSFORM_FWD && mode != E2EG_TRANSFORM_BWD)
        return fail(E2EG_ERR_INVALID_ARG, "%s: mode %d", who, mode);
    if (dtype != E2EG_BF16)
        return fail(E2EG_ERR_BAD_DTYPE, "%s: only E2EG_BF16 is supported (got %d)", who, dtype);
    if (n < 0) return fail(E2EG_ERR_INVALID_ARG, "%s: negative n", who);
    if (Fin <= 0 || Fout <= 0 || Fin % 32 || Fout % 32 || Fin > kMaxF || Fout > kMaxF)
        return fail(E2EG_ERR_INVALID_ARG, "%s: Fin=%d, Fout=%d must be multiples of 32 in [32, %d]", who, Fin,
                    Fout, kMaxF);
    if (!d_P || !d_W || !d_H) return fail(E2EG_ERR_NULL_PTR, "%s: d_P, d_W or d_H is null", who);
    if (mode == E2EG_TRANSFORM_BWD && !d_gH) return fail(E2EG_ERR_NULL_PTR, "%s: d_gH is null", who);
    const void* ptrs[] = {d_P, d_W, d_H, d_gH, d_gP, d_gW};
    for (const void* q : ptrs)
        if (q && !aligned_to(q, 16)) return fail(E2EG_ERR_INVALID_ARG, "%s: a pointer is not 16-byte aligned", who);
    const size_t need = e2eg_layer_transform_workspace_bytes(mode, n, Fin, Fout, dtype);
    if (static_scratch && E2EG_TRANSFORM_STATIC_SCRATCH_BYTES < need)
        return fail(E2EG_ERR_CAPACITY, "%s: n=%d, Fin=%d, Fout=%d need %zu bytes of scratch memory, the static array "
                                       "holds %zu; use e2eg_layer_transform with a workspace", who, n, Fin, Fout, need,
                    (size_t)E2EG_TRANSFORM_STATIC_SCRATCH_BYTES);
    if (static_scratch) {   // arguments are fine: now the array's address on this device
        float* ptr = nullptr;
        const int32_t st = static_scratch_of_current_device(&ptr);
        if (st != E2EG_OK) return st;
        ws = ptr;
        ws_bytes = E2EG_TRANSFORM_STATIC_SCRATCH_BYTES;
    }
    if (!ws || !aligned_to(ws, kAlign) || ws_bytes < need)
        return fail(E2EG_ERR_WORKSPACE, "%s: workspace needs %zu bytes, 256-byte aligned", who, need);
    hipStream_t stream = static_cast<hipStream_t>(stream_);

    if (mode == E2EG_TRANSFORM_FWD) {
        if (n == 0) return E2EG_OK;
        if (relu) launch_dense<false, true, true>(d_P, nullptr, d_W, d_H, n, Fin, Fout, Fout, stream);
        else launch_dense<false, true, false>(d_P, nullptr, d_W, d_H, n, Fin, Fout, Fout, stream);
        E2EG_LAUNCH_CHECK("dense_rows");
        return E2EG_OK;
    }
    if (d_gP && n > 0) {
        if (relu) launch_dense<true, false, false>(d_gH, d_H, d_W, d_gP, n, Fout, Fin, Fout, stream);
        else launch_dense<false, false, false>(d_gH, nullptr, d_W, d_gP, n, Fout, Fin, Fout, stream);
        E2EG_LAUNCH_CHECK("dense_rows");
    }
    if (d_gW) {
        const int32_t rpb = rows_per_block_for(n);
        const int32_t blocks = n > 0 ? (int32_t)ceil_div(n, rpb) : 0;
        float* partial = static_cast<float*>(ws);
        if (blocks > 0) {
            const dim3 grid((unsigned)blocks, (unsigned)ceil_div(Fin, 128), (unsigned)ceil_div(Fout, 128));
            const uint16_t* p = static_cast<const uint16_t*>(d_P);
            const uint16_t* gh = static_cast<const uint16_t*>(d_gH);
            const uint16_t* h = static_cast<const uint16_t*>(d_H);
            if (relu) weight_grad_partial<true><<<grid, dim3(kThreads), 0, stream>>>(p, gh, h, partial, n, Fin, Fout, rpb);
            else weight_grad_partial<false><<<grid, dim3(kThreads), 0, stream>>>(p, gh, h, partial, n, Fin, Fout, rpb);
            E2EG_LAUNCH_CHECK("weight_grad_partial");
        }
        const int32_t count = Fin * Fout;
        weight_grad_reduce<<<dim3((unsigned)ceil_div(count, kReduceElems)), dim3(kThreads), 0, stream>>>(partial, blocks, count, d_gW);
        E2EG_LAUNCH_CHECK("weight_grad_reduce");
    }
    return E2EG_OK;
}
}  // namespace

extern "C" int32_t e2eg_layer_transform(int32_t mode, int32_t n, int32_t Fin, int32_t Fout,
                                        int32_t dtype, int32_t relu, const void* d_P,
                                        const void* d_W, void* d_H, const void* d_gH, void* d_gP,
                                        float* d_gW, void* ws, size_t ws_bytes, void* stream) {
    return transform_impl("layer_transform", false, mode, n, Fin, Fout, dtype, relu, d_P, d_W, d_H, d_gH, d_gP, d_gW, ws,
                          ws_bytes, stream);
}

extern "C" int32_t e2eg_layer_transform_noalloc(int32_t mode, int32_t n, int32_t Fin, int32_t Fout, int32_t dtype,
                                                int32_t relu, const void* d_P, const void* d_W, void* d_H,
                                                const void* d_gH, void* d_gP, float* d_gW, void* stream) {
    // every partial matrix the reduction reads is written in full by the kernel before it, so the
    // array's old contents (the previous call's) never show and nothing has to be cleared
    return transform_impl("layer_transform_noalloc", true, mode, n, Fin, Fout, dtype, relu, d_P, d_W, d_H, d_gH, d_gP,
                          d_gW, nullptr, 0, stream);
}
