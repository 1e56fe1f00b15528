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

constexpr int kDenseWaves = 8;               // wavefronts per workgroup of dense_rows (4 where a row has more than 8 k-steps
                                             // and a wavefront needs more than 256 registers): they share one weight tile
constexpr int kDenseDepth = 1;               // tiles a wavefront of dense_rows requests ahead (2 measured slower: 25.4 against
                                             // 23.3 us at 200 k rows, 408 against 392 us at 4 M)
constexpr int kGradWaves = 8;                // wavefronts per workgroup of weight_grad_partial
constexpr int kGradThreads = 64 * kGradWaves;
constexpr int kReduceThreads = 256;
constexpr int kMaxF = 256;
constexpr int kDenseMaxGroups = 256;         // workgroups of 8 wavefronts of dense_rows per column group: their registers
                                             // allow one per compute unit
constexpr int kPad = 8;                      // LDS row padding (elements) against bank conflicts
constexpr int kWeightLds = 128 * (128 + kPad);  // elements; also fits 64 x (256 + kPad)
constexpr int kOutLd = 128 + kPad;           // pitch of a wavefront's result rows in LDS (at most 128 columns per workgroup)
constexpr int kTileRows = 128;               // node rows per step of the dW kernel
constexpr int kPairPasses = kTileRows / 64;  // a thread stages one pair of rows of every 32 pairs ...
constexpr int kChunkLanes = kGradThreads / 32;        // ... and one 8-column chunk of every kChunkLanes
constexpr int kChunkReps = 16 / kChunkLanes;          // (a 128-column tile has 16 chunks)
constexpr int kGradOSplit = kGradWaves / 4;  // wavefronts that share a 32-column block of P split the dZ columns
constexpr int kGradOBlocks = 4 / kGradOSplit;
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
// grid.x: workgroups that each take `tiles` blocks of 32 WAVES rows, block b + t * gridDim.x in
// turn t, so that at any moment the workgroups in flight read and write one moving stretch of the
// tables (the weight tile is staged once per workgroup and serves all its turns); grid.y: groups of
// `ngroup` output columns.
// KS: the most k-steps of 16 a row can have (8 for up to 128 input columns).  A wavefront requests
// the rows of its next kDenseDepth tiles before it multiplies the current one, so that the loads
// overlap the staging of the weights, the product and the stores.
// EXACT: kdim == 16 * KS and every workgroup has 128 output columns, so that the loops over
// k-steps and column blocks have constant bounds and compile to straight-line code.
template <bool MASKED, bool TRANS_W, bool RELU, int KS, bool EXACT, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void dense_rows(const uint16_t* __restrict__ a_rows,
                                                       const uint16_t* __restrict__ mask_rows,
                                                       const uint16_t* __restrict__ w,
                                                       uint16_t* __restrict__ out, int32_t n,
                                                       int32_t kdim, int32_t ndim, int32_t w_ld,
                                                       int32_t ngroup, int32_t tiles, int32_t stream_out) {
    __shared__ __attribute__((aligned(16))) uint16_t bt[kWeightLds];  // [ngroup][kdim + kPad]
    __shared__ __attribute__((aligned(16))) uint16_t ot[WAVES][16 * kOutLd];  // per wavefront: 16 result rows
    // The weight tile: k contiguous per output column, rows padded by kPad elements, which spreads a
    // wavefront's 16-byte reads of 32 columns over the banks.  (An unpadded tile with the 16-byte groups of
    // column c stored at group index ^ (c + c / 8) % 8 was measured too: SQ_LDS_BANK_CONFLICT 0.55 of the
    // LDS cycles against 0.23 for the padding.)
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
    constexpr int kDenseThreads = 64 * WAVES;
    constexpr int kRowsPerBlock = 32 * WAVES;   // one 32-row MFMA tile per wavefront
    const int64_t row_first = (int64_t)blockIdx.x * kRowsPerBlock + wave * 32 + l32;
    const int64_t row_step = (int64_t)gridDim.x * kRowsPerBlock;
    // tiles requested ahead of the one being multiplied (each holds KS, masked 2 KS, 16-byte registers)
    constexpr int DEPTH = (MASKED || KS > 8) ? 1 : kDenseDepth;
    uint4 nxt_a[DEPTH][KS], nxt_m[DEPTH][MASKED ? KS : 1];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) load_rows(row_first + d * row_step, nxt_a[d], nxt_m[d]);   // in flight while the weight tile is staged
    if (TRANS_W) {
        // Transposing.  A thread takes the same 8 columns of two consecutive rows of W (k = 2 kp, 2 kp + 1),
        // 16 bytes each, and writes, for each of the 8 columns, the pair as one 4-byte word into that
        // column's row of the tile.  Consecutive lanes hold consecutive kp: a store instruction fills
        // consecutive banks.
        const int cvecs = ng / 8, kpairs = kdim / 2;
        uint32_t* bt32 = reinterpret_cast<uint32_t*>(bt);
        const int ldw = ldb / 2;
        for (int e = threadIdx.x; e < kpairs * cvecs; e += kDenseThreads) {
            const int ch = e / kpairs, kp = e - ch * kpairs;
            const uint16_t* src = w + (int64_t)(2 * kp) * w_ld + n0 + ch * 8;
            const uint4 q0 = *reinterpret_cast<const uint4*>(src);
            const uint4 q1 = *reinterpret_cast<const uint4*>(src + w_ld);
            const uint32_t w0[4] = {q0.x, q0.y, q0.z, q0.w};
            const uint32_t w1[4] = {q1.x, q1.y, q1.z, q1.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = ch * 8 + 2 * j;
                bt32[c * ldw + kp] = (w0[j] & 0xffffu) | (w1[j] << 16);
                bt32[(c + 1) * ldw + kp] = (w0[j] >> 16) | (w1[j] & 0xffff0000u);
            }
        }
    } else {
        const int kvecs = kdim / 8;
        for (int e = threadIdx.x; e < ng * kvecs; e += kDenseThreads) {
            const int c = e / kvecs, kv = e - c * kvecs;
            *reinterpret_cast<uint4*>(bt + c * ldb + kv * 8) =
                *reinterpret_cast<const uint4*>(w + (int64_t)(n0 + c) * w_ld + kv * 8);
        }
    }
    __syncthreads();

#pragma unroll 1
    for (int tile = 0; tile < tiles; ++tile) {
    const int64_t row = row_first + tile * row_step;
    if ((int64_t)row - l32 >= n) return;   // the whole wavefront is past the end

    uint4 areg[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) areg[ks] = MASKED ? mask_vec(nxt_a[0][ks], nxt_m[0][ks]) : nxt_a[0][ks];
#pragma unroll
    for (int d = 0; d + 1 < DEPTH; ++d) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            nxt_a[d][ks] = nxt_a[d + 1][ks];
            if (MASKED) nxt_m[d][ks] = nxt_m[d + 1][ks];
        }
    }
    if (tile + DEPTH < tiles) load_rows(row + DEPTH * row_step, nxt_a[DEPTH - 1], nxt_m[DEPTH - 1]);
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
// The node rows are the contraction index, so both operands go through LDS transposed, kTileRows rows a
// step.  A thread takes the same 8 columns of two consecutive rows and writes, for each column, the pair as
// one 4-byte word: consecutive lanes hold consecutive row pairs, so a store instruction fills consecutive
// banks.  The rows of the next two steps are requested while the current one is multiplied.
template <bool MASKED>
__global__ __launch_bounds__(kGradThreads) void weight_grad_partial(const uint16_t* __restrict__ p,
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
    const int rp = threadIdx.x & 31;   // row pair of the tile (and every 32nd after it)
    const int cq = threadIdx.x >> 5;   // 8-column chunk (and every kChunkLanes-th after it)
    const int oblocks = og / 32;
    // products: this wavefront owns 32 columns of P and kGradOBlocks blocks of 32 columns of dZ
    const int cw = wave & 3;
    const int ob0 = (wave >> 2) * kGradOBlocks;
    const bool wave_live = cw * 32 < cg && ob0 < oblocks;

    f32x16 acc[kGradOBlocks];
#pragma unroll
    for (int ob = 0; ob < kGradOBlocks; ++ob)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[ob][i] = 0.0f;

    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r_end = r_begin + rows_per_block < n ? r_begin + rows_per_block : n;
    // A thread's pieces of one step: for each of its row pairs and column chunks, two rows of P and of dZ
    // (dZ with its mask still beside it).  Piece i: chunk rep i % kChunkReps, pair pass i / kChunkReps.
    constexpr int kPieces = kChunkReps * kPairPasses;
    struct Step {
        uint4 p0[kPieces], p1[kPieces], z0[kPieces], z1[kPieces], h0[MASKED ? kPieces : 1], h1[MASKED ? kPieces : 1];
    };
    auto load_step = [&](Step& q, int64_t r0) {
#pragma unroll
        for (int i = 0; i < kPieces; ++i) {
            const int cv = cq + (i % kChunkReps) * kChunkLanes;
            const int64_t r = r0 + 2 * (rp + (i / kChunkReps) * 32);
            const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
            q.p0[i] = q.p1[i] = q.z0[i] = q.z1[i] = zero;
            if (MASKED) q.h0[i] = q.h1[i] = zero;
            if (r < r_end) {
                if (cv * 8 < cg) q.p0[i] = *reinterpret_cast<const uint4*>(p + r * fin + c0 + cv * 8);
                if (cv * 8 < og) {
                    q.z0[i] = *reinterpret_cast<const uint4*>(gh + r * fout + o0 + cv * 8);
                    if (MASKED) q.h0[i] = *reinterpret_cast<const uint4*>(h + r * fout + o0 + cv * 8);
                }
            }
            if (r + 1 < r_end) {
                if (cv * 8 < cg) q.p1[i] = *reinterpret_cast<const uint4*>(p + (r + 1) * fin + c0 + cv * 8);
                if (cv * 8 < og) {
                    q.z1[i] = *reinterpret_cast<const uint4*>(gh + (r + 1) * fout + o0 + cv * 8);
                    if (MASKED) q.h1[i] = *reinterpret_cast<const uint4*>(h + (r + 1) * fout + o0 + cv * 8);
                }
            }
        }
    };
    uint32_t* pt32 = reinterpret_cast<uint32_t*>(pt);
    uint32_t* zt32 = reinterpret_cast<uint32_t*>(zt);
    constexpr int kTileLdw = kTileLd / 2;
    auto write_pairs = [&](uint32_t* t32, int cv, int pair, const uint4 a, const uint4 b) {
        const uint32_t wa[4] = {a.x, a.y, a.z, a.w};
        const uint32_t wb[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            t32[(cv * 8 + 2 * j) * kTileLdw + pair] = (wa[j] & 0xffffu) | (wb[j] << 16);
            t32[(cv * 8 + 2 * j + 1) * kTileLdw + pair] = (wa[j] >> 16) | (wb[j] & 0xffff0000u);
        }
    };
    // one step: its rows into the tiles, the step after next requested into the registers just freed, product
    auto do_step = [&](Step& q, int64_t r_next) {
#pragma unroll
        for (int i = 0; i < kPieces; ++i) {
            const int cv = cq + (i % kChunkReps) * kChunkLanes;
            const int pair = rp + (i / kChunkReps) * 32;
            write_pairs(pt32, cv, pair, q.p0[i], q.p1[i]);
            write_pairs(zt32, cv, pair, MASKED ? mask_vec(q.z0[i], q.h0[i]) : q.z0[i],
                        MASKED ? mask_vec(q.z1[i], q.h1[i]) : q.z1[i]);
        }
        __syncthreads();
        if (r_next < r_end) load_step(q, r_next);
        if (wave_live) {
#pragma unroll
            for (int ks = 0; ks < kTileRows / 16; ++ks) {
                const uint4 a = *reinterpret_cast<const uint4*>(pt + (cw * 32 + l32) * kTileLd + ks * 16 + khalf * 8);
#pragma unroll
                for (int ob = 0; ob < kGradOBlocks; ++ob) {
                    if (ob0 + ob < oblocks) {
                        const uint4 b = *reinterpret_cast<const uint4*>(zt + ((ob0 + ob) * 32 + l32) * kTileLd + ks * 16 + khalf * 8);
                        acc[ob] = mfma(a, b, acc[ob]);  // D[c][o]
                    }
                }
            }
        }
        __syncthreads();
    };
    Step qa, qb;
    load_step(qa, r_begin);
    load_step(qb, r_begin + kTileRows);   // past r_end: zeros, nothing read
    for (int64_t r0 = r_begin; r0 < r_end; r0 += 2 * kTileRows) {
        do_step(qa, r0 + 2 * kTileRows);
        if (r0 + kTileRows < r_end) do_step(qb, r0 + 3 * kTileRows);
    }
    if (!wave_live) return;
    float* dst = partial + (int64_t)blockIdx.x * fin * fout;
#pragma unroll
    for (int ob = 0; ob < kGradOBlocks; ++ob) {
        if (ob0 + ob < oblocks) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int c = c0 + cw * 32 + (i / 4) * 8 + khalf * 4 + (i % 4);
                dst[(int64_t)c * fout + o0 + (ob0 + ob) * 32 + l32] = acc[ob][i];
            }
        }
    }
}

// gw[e] = sum over blocks of partial[b][e], in double and in a fixed order: thread (q, j) of a
// workgroup adds blocks q, q + 8, q + 16, ... for element e0 + j; the eight sums of an element are
// then added in q order.
constexpr int kReduceElems = 32;   // elements per workgroup (one 128-byte line of every partial matrix)
constexpr int kReduceSlices = kReduceThreads / kReduceElems;

__global__ __launch_bounds__(kReduceThreads) void weight_grad_reduce(const float* __restrict__ partial, int32_t nblocks,
                                                               int32_t count, float* __restrict__ gw) {
    __shared__ double red[kReduceSlices][kReduceElems];
    const int j = threadIdx.x % kReduceElems, q = threadIdx.x / kReduceElems;
    const int e = blockIdx.x * kReduceElems + j;
    double s = 0.0;
    if (e < count) {
#pragma unroll 16
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
    r = (r + 63) / 64 * 64;
    return (int32_t)(r < 128 ? 128 : r);
}

template <bool MASKED, bool TRANS_W, bool RELU, int KS, bool EXACT, int WAVES>
void launch_dense_as(const void* a, const void* mask, const void* w, void* out, int32_t n, int32_t kdim, int32_t ndim,
                     int32_t w_ld, int32_t ngroup, hipStream_t stream) {
    // eight wavefronts per compute unit, each taking as many tiles in turn as that leaves it, but no more
    // workgroups than blocks of rows
    const int64_t blocks = ceil_div(n, (int64_t)32 * WAVES);
    int64_t tiles = ceil_div(blocks, (int64_t)kDenseMaxGroups * (8 / WAVES));
    tiles = tiles < 1 ? 1 : tiles;
    const dim3 grid((unsigned)ceil_div(blocks, tiles), (unsigned)ceil_div(ndim, ngroup));
    // streaming stores once the result is far larger than the caches (measured: 5 % at 4 M rows); below
    // that the next kernel of a mini-batch step finds the rows in the caches if they are written normally
    const int32_t stream_out = (int64_t)n * ndim * 2 > (64ll << 20) ? 1 : 0;
    dense_rows<MASKED, TRANS_W, RELU, KS, EXACT, WAVES><<<grid, dim3(64 * WAVES), 0, stream>>>(
        static_cast<const uint16_t*>(a), static_cast<const uint16_t*>(mask), static_cast<const uint16_t*>(w),
        static_cast<uint16_t*>(out), n, kdim, ndim, w_ld, ngroup, (int32_t)tiles, stream_out);
}

template <bool MASKED, bool TRANS_W, bool RELU>
void launch_dense(const void* a, const void* mask, const void* w, void* out, int32_t n, int32_t kdim,
                  int32_t ndim, int32_t w_ld, hipStream_t stream) {
    const int32_t ngroup = kdim > 128 ? 64 : 128;
    if (kdim == 128 && ndim % 128 == 0)
        launch_dense_as<MASKED, TRANS_W, RELU, 8, true, kDenseWaves>(a, mask, w, out, n, kdim, ndim, w_ld, ngroup, stream);
    else if (kdim <= 128)
        launch_dense_as<MASKED, TRANS_W, RELU, 8, false, kDenseWaves>(a, mask, w, out, n, kdim, ndim, w_ld, ngroup, stream);
    else
        launch_dense_as<MASKED, TRANS_W, RELU, kMaxF / 16, false, 4>(a, mask, w, out, n, kdim, ndim, w_ld, ngroup, stream);
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
            if (relu) weight_grad_partial<true><<<grid, dim3(kGradThreads), 0, stream>>>(p, gh, h, partial, n, Fin, Fout, rpb);
            else weight_grad_partial<false><<<grid, dim3(kGradThreads), 0, stream>>>(p, gh, h, partial, n, Fin, Fout, rpb);
            E2EG_LAUNCH_CHECK("weight_grad_partial");
        }
        const int32_t count = Fin * Fout;
        weight_grad_reduce<<<dim3((unsigned)ceil_div(count, kReduceElems)), dim3(kReduceThreads), 0, stream>>>(partial, blocks, count, d_gW);
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
