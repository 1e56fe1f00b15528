// e2eg_propagate_fwd / e2eg_propagate_bwd: K layers of H(l+1) = A^ H(l) with
// A^ = D~^-1/2 (A + I) D~^-1/2 (paper: Section 3 "Notation"; Section 3.1, LightGCN matrix
// form) and the transposed pass G(l) = A^T G(l+1) (Appendix A, "GNN backprop" factor).
//
// How the GPU evaluates it.  With s = d~^-1/2 and Z(l) = S H(l) (rows pre-scaled by s),
//     H(l+1) = S * (A~ Z(l)),        Z(l+1) = S * H(l+1),
// so a layer is an UNWEIGHTED sum of neighbour rows of Z followed by one scale per output row: the
// only per-edge datum read is the 4-byte column index.  Z(0) is made by one streaming pre-scale
// pass; every later Z(l) is written by the layer that produces it.  Layers the caller asked for are
// stored as H(l); layers it did not ask for exist only as Z(l).  Every Z buffer carries one extra
// all-zero row (index n): "no neighbour" lanes read it, which keeps the gather loop free of
// per-lane predicates.
// Where the pre-scale pass would cost as much as the work it prepares (a single-layer call, a
// small graph) the first layer instead gathers the caller's rows H(0) directly, by node id, and
// multiplies each by s_j, both read from the schedule beside each other (kFirst below; a lane
// without a neighbour then gathers its row's first neighbour again with weight 0, the caller's table
// having no zero row).
//
// Kernel shape (wave64).  The kernels read the renumbered copy of the graph that e2eg_normalize
// leaves in the schedule ("internal" ids, see common.h); Z buffers are in internal row order, H
// is written by node id.  A group of G = 16-byte-chunks-per-row lanes reads one neighbour row
// with 16-byte loads, so one load instruction of a wavefront fetches 64/G neighbour rows; eight
// such instructions are in flight per lane.  Byte offsets are 32-bit (one v_mad_u32_u24 per
// gather on a scalar base address) and "no neighbour" lanes read the zero row, so the loop has
// no per-lane predicate; bf16 results are packed by v_cvt_pk_bf16_f32.
//   - Rows of more than kShortMax entries: all 64 lanes work on one row (or on one segment of at
//     most kSegLen entries of it), the 64/G lane groups taking different neighbours; their sums are
//     added across lanes at the end.  A row of several segments leaves fp32 partial sums that a
//     second kernel adds in a fixed order (in double): no floating-point atomics, results are
//     reproducible.
//   - Short rows: 64/G rows side by side, one lane group per row.  Nothing is summed across
//     lanes, and the per-row work (bounds, scale, conversion, store) is paid once per 64/G rows;
//     on a power-law graph most rows are short and this per-row work, not memory, was what bound
//     the first version of the kernel (vector-ALU issue).
// On a weighted graph (e2eg_propagate_weighted_*) the schedule also holds the entries' values, in
// the order of its own column indices; the instantiations that carry a value per entry (kValues:
// inner layers of a weighted graph; kFirst: the first layer of any graph) load it beside the
// index (same predicates), hand it to the lanes by the same shuffles, and replace the add of a
// gathered row by a multiply-add.  e2eg_aggregate is the kernel of the inner layers on a table
// pre-scaled by a streaming pass, with other per-row scales (mean, transposed mean, plain sum) and
// an optional addend.
// Measured on gfx950: the dot-product instruction v_dot2c_f32_bf16 with unit weights adds a
// bf16 pair in one instruction instead of shift + add per element, but ran slower than the plain
// sequence, and capping registers for more resident wavefronts cost more in spills than it gained;
// neither is used.
#include "common.h"

#include <type_traits>

namespace e2eg {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// ---- storage types ---------------------------------------------------------------------------
struct F32 {
    using elem = float;
    static constexpr int kVec = 4;  // elements per 16 bytes
};
struct BF16 {
    using elem = uint16_t;
    static constexpr int kVec = 8;
};

__device__ __forceinline__ float bf16_to_f32(uint32_t bits) { return __uint_as_float(bits << 16); }

// Two floats -> packed bf16, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

template <typename T>
__device__ __forceinline__ void load_vec(const typename T::elem* p, float (&v)[T::kVec]);
template <>
__device__ __forceinline__ void load_vec<F32>(const float* p, float (&v)[4]) {
    const float4 q = *reinterpret_cast<const float4*>(p);
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
}
template <>
__device__ __forceinline__ void load_vec<BF16>(const uint16_t* p, float (&v)[8]) {
    const uint4 q = *reinterpret_cast<const uint4*>(p);
    v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
    v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
    v[4] = __uint_as_float(q.z << 16); v[5] = __uint_as_float(q.z & 0xffff0000u);
    v[6] = __uint_as_float(q.w << 16); v[7] = __uint_as_float(q.w & 0xffff0000u);
}

// Layer outputs and partial sums are written once and not read again by the same kernel.  `stream`
// (wave-uniform): write them with streaming stores, which keeps them from displacing the feature rows
// the gathers reuse in L2 - right when the tables are far larger than the caches (1 % on the 50 M-edge
// graph).  On a small graph the next kernel finds them in the caches if they are written normally
// (4.5 % on the 2 M-edge graph), so there `stream` is off; launch_layer decides by the table's size.
template <typename T>
__device__ __forceinline__ void store_vec(typename T::elem* p, const float (&v)[T::kVec], bool stream);
template <>
__device__ __forceinline__ void store_vec<F32>(float* p, const float (&v)[4], bool stream) {
    const f32x4 q = {v[0], v[1], v[2], v[3]};
    if (stream) __builtin_nontemporal_store(q, reinterpret_cast<f32x4*>(p));
    else *reinterpret_cast<f32x4*>(p) = q;
}
template <>
__device__ __forceinline__ void store_vec<BF16>(uint16_t* p, const float (&v)[8], bool stream) {
    const u32x4 q = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
    if (stream) __builtin_nontemporal_store(q, reinterpret_cast<u32x4*>(p));
    else *reinterpret_cast<u32x4*>(p) = q;
}

template <typename T>
__device__ __forceinline__ float load_one(const typename T::elem* p);
template <>
__device__ __forceinline__ float load_one<F32>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float load_one<BF16>(const uint16_t* p) { return bf16_to_f32(*p); }

template <typename T>
__device__ __forceinline__ void store_one(typename T::elem* p, float v);
template <>
__device__ __forceinline__ void store_one<F32>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_one<BF16>(uint16_t* p, float v) { *p = (uint16_t)(pack_bf16(v, 0.0f) & 0xffffu); }

// ---- one layer --------------------------------------------------------------------------------
template <typename T>
struct LayerArgs {
    const float* dinv_sqrt;       // by node id
    SchedView sched;              // internal graph (see common.h)
    const typename T::elem* zin;  // Z(l) = S H(l), [n + 1][F] in internal order, row n all zero; kFirst: H(0) by node id
    int64_t ld_in;                // leading dimension of zin in elements (F for a Z buffer)
    const int32_t* cols;          // column of every entry: zcol (rows of Z), or znode for kFirst
    const float* vals;            // value of every entry: null (kPlain), zval (kValues), zs (kFirst)
    int32_t transposed;           // the call computes with the transpose of the stored operator
    int32_t stream_out;           // results leave through streaming stores (tables far larger than the caches)
    typename T::elem* out_h;      // H(l+1) by node id, or null
    int64_t ld_h;
    typename T::elem* out_z;      // Z(l+1) = S H(l+1), [n + 1][F] in internal order, or null
    const typename T::elem* addend;  // direct term added to H(l+1) before scaling (by node id), or null
    int64_t ld_add;
    float* partial;               // [slots][F] fp32
    int32_t F;
    int32_t n;                    // also the index of the zero row
    int32_t a_blocks;             // workgroups per XCD the launch provides for slotted segments
    int32_t b_blocks;             // workgroups per XCD for rows of one segment
};

// What a gathered row is multiplied by: nothing (inner layers), the entry's value (inner layers of a
// weighted graph), or s_j times that value while the rows come from the caller's H(0) (first layer).
constexpr int kPlain = 0, kValues = 1, kFirst = 2;

// The backward entry points apply the stored operator itself, which is its transpose only if structure
// and values are symmetric; a schedule that e2eg_normalize found not to be is refused on the device,
// without a read-back: every row scale, and so every result, is NaN.  Decided once per wavefront, at
// the start of the kernel (a scalar load inside the row loops would wait for the cross-lane moves in
// flight with it).
template <typename T>
__device__ __forceinline__ bool refused(const LayerArgs<T>& a) {
    return a.transposed && a.sched.header->flags != 0;
}
template <typename T>
__device__ __forceinline__ float row_scale(const LayerArgs<T>& a, int32_t node, bool refuse) {
    return refuse ? __builtin_nanf("") : a.dinv_sqrt[node];
}

// Accumulators of one lane: acc[v] holds this lane's 16-byte chunk as fp32.
template <typename T>
struct Sum {
    float acc[T::kVec];
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int v = 0; v < T::kVec; ++v) acc[v] = 0.0f;
    }
    __device__ __forceinline__ void add(const uint4 q) {
        if constexpr (std::is_same<T, F32>::value) {
            acc[0] += __uint_as_float(q.x); acc[1] += __uint_as_float(q.y);
            acc[2] += __uint_as_float(q.z); acc[3] += __uint_as_float(q.w);
        } else {
            acc[0] += __uint_as_float(q.x << 16); acc[1] += __uint_as_float(q.x & 0xffff0000u);
            acc[2] += __uint_as_float(q.y << 16); acc[3] += __uint_as_float(q.y & 0xffff0000u);
            acc[4] += __uint_as_float(q.z << 16); acc[5] += __uint_as_float(q.z & 0xffff0000u);
            acc[6] += __uint_as_float(q.w << 16); acc[7] += __uint_as_float(q.w & 0xffff0000u);
        }
    }
    // acc += w * chunk (weighted graphs: w is the value of the CSR entry)
    __device__ __forceinline__ void add_scaled(const uint4 q, const float w) {
        if constexpr (std::is_same<T, F32>::value) {
            acc[0] = fmaf(w, __uint_as_float(q.x), acc[0]); acc[1] = fmaf(w, __uint_as_float(q.y), acc[1]);
            acc[2] = fmaf(w, __uint_as_float(q.z), acc[2]); acc[3] = fmaf(w, __uint_as_float(q.w), acc[3]);
        } else {
            acc[0] = fmaf(w, __uint_as_float(q.x << 16), acc[0]); acc[1] = fmaf(w, __uint_as_float(q.x & 0xffff0000u), acc[1]);
            acc[2] = fmaf(w, __uint_as_float(q.y << 16), acc[2]); acc[3] = fmaf(w, __uint_as_float(q.y & 0xffff0000u), acc[3]);
            acc[4] = fmaf(w, __uint_as_float(q.z << 16), acc[4]); acc[5] = fmaf(w, __uint_as_float(q.z & 0xffff0000u), acc[5]);
            acc[6] = fmaf(w, __uint_as_float(q.w << 16), acc[6]); acc[7] = fmaf(w, __uint_as_float(q.w & 0xffff0000u), acc[7]);
        }
    }
    // `live` of the U gathered chunks q[0..U) are valid (wave-uniform count)
    template <int U>
    __device__ __forceinline__ void add_batch(const uint4 (&q)[U], int live) {
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (u < live) add(q[u]);
    }
    template <int U>
    __device__ __forceinline__ void add_batch_scaled(const uint4 (&q)[U], const float (&w)[U], int live) {
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (u < live) add_scaled(q[u], w[u]);
    }

    // -> out[] = the chunk's total over the lane groups, valid in lanes of group 0
    template <int LOG_G>
    __device__ __forceinline__ void total(float (&out)[T::kVec]) {
#pragma unroll
        for (int off = 1 << LOG_G; off < 64; off <<= 1) {
#pragma unroll
            for (int v = 0; v < T::kVec; ++v) acc[v] += __shfl_xor(acc[v], off);
        }
#pragma unroll
        for (int v = 0; v < T::kVec; ++v) out[v] = acc[v];
    }
};

// Per-row finish: h = s * sum (+ addend); store H (by node id) and/or Z = s * h (internal row).
template <typename T>
__device__ __forceinline__ void finish_vec(const LayerArgs<T>& a, int32_t zrow, int32_t node, float s,
                                           int32_t col, float (&acc)[T::kVec]) {
    float h[T::kVec];
#pragma unroll
    for (int v = 0; v < T::kVec; ++v) h[v] = s * acc[v];
    if (a.addend) {
        float d[T::kVec];
        load_vec<T>(a.addend + (int64_t)node * a.ld_add + col, d);
#pragma unroll
        for (int v = 0; v < T::kVec; ++v) h[v] += d[v];
    }
    if (a.out_h) store_vec<T>(a.out_h + (int64_t)node * a.ld_h + col, h, a.stream_out != 0);
    if (a.out_z) {
#pragma unroll
        for (int v = 0; v < T::kVec; ++v) h[v] *= s;
        store_vec<T>(a.out_z + (int64_t)zrow * a.F + col, h, a.stream_out != 0);
    }
}

// 16 bytes of row j at byte offset `lane_off` inside the row.  NARROW: the table is below 4 GiB
// and has fewer than 2^24 rows, so the offset is one 24-bit multiply-add on a scalar base.
template <typename T, bool NARROW>
__device__ __forceinline__ uint4 gather16(const LayerArgs<T>& a, int32_t j, uint32_t row_bytes,
                                          uint32_t lane_off) {
    const char* base = reinterpret_cast<const char*>(a.zin);
    if constexpr (NARROW) {
        return *reinterpret_cast<const uint4*>(base + (__umul24((uint32_t)j, row_bytes) + lane_off));
    } else {
        return *reinterpret_cast<const uint4*>(base + ((uint64_t)(uint32_t)j * row_bytes + lane_off));
    }
}

constexpr int kInFlight = 8;  // independent 16-byte gathers in flight per lane
// The column indices (and entry values) are streamed once, but they are read with ordinary loads:
// measured, non-temporal loads for them cost 6 % (500 M-edge graph, 128-byte rows) to 9 % (2 M-edge
// fp32 graph) of a launch.

// One segment (entries [beg, end) of internal row seg.row, at most kSegLen of them), all 64 lanes
// on the one row: G lanes per neighbour row, 64/G neighbour rows per load instruction.  Column
// indices are fetched 64 at a time, one coalesced load, the next 64 requested before the current
// gathers are consumed.  slot >= 0: the sum goes to that partial-sum slot; slot < 0: the segment is
// the whole row and the row is finished here.
template <typename T, int LOG_G, bool NARROW, int MODE>
__device__ __forceinline__ void run_segment(const LayerArgs<T>& a, const Segment seg, const int lane,
                                            const bool refuse) {
    constexpr int G = 1 << LOG_G;
    constexpr int NB = 64 >> LOG_G;
    constexpr int V = T::kVec;
    constexpr int U = kInFlight;
    constexpr bool VALS = MODE != kPlain;
    const int g = lane >> LOG_G;
    const int c = lane & (G - 1);
    const int chunks = a.F / V;
    const uint32_t row_bytes = (uint32_t)a.ld_in * (uint32_t)sizeof(typename T::elem);
    int32_t node = 0;
    float s = 0.0f;
    if (seg.slot < 0) {  // requested now, needed after the gathers
        node = a.sched.orig[seg.row];
        s = row_scale<T>(a, node, refuse);
    }
    // What a lane without a neighbour gathers: the all-zero row of a Z buffer; kFirst, whose table has
    // no such row: the segment's own first neighbour, with weight 0 (adds 0, and NaN only where that
    // neighbour makes the sum NaN anyway).
    int32_t idx_first = lane < seg.end - seg.beg ? *(a.cols + seg.beg + lane) : a.n;
    const int32_t none = MODE == kFirst ? __builtin_amdgcn_readfirstlane(idx_first) : a.n;
    if constexpr (MODE == kFirst)
        if (lane >= seg.end - seg.beg) idx_first = none;
    float wgt_first = 0.0f;  // VALS: the entries' values travel with their column indices
    if constexpr (VALS)
        if (lane < seg.end - seg.beg) wgt_first = *(a.vals + seg.beg + lane);

    for (int cb = 0; cb < chunks; cb += G) {   // more than one pass only for rows wider than 1 KiB
        const int cc = cb + c;
        const bool active = cc < chunks;       // idle lanes re-read chunk 0; their sums are dropped
        const uint32_t lane_off = active ? (uint32_t)cc * 16u : 0u;
        Sum<T> sum;
        sum.clear();
        int32_t idx = idx_first;
        float wgt = wgt_first;
        for (int32_t base = seg.beg; base < seg.end; base += 64) {
            const int cnt = seg.end - base < 64 ? seg.end - base : 64;
            int32_t idx_next = none;
            float wgt_next = 0.0f;
            if (base + 64 < seg.end && lane < seg.end - base - 64) {
                idx_next = *(a.cols + base + 64 + lane);
                if constexpr (VALS) wgt_next = *(a.vals + base + 64 + lane);
            }
            int t = 0;
            for (; t + U * NB <= cnt; t += U * NB) {   // full batches: every lane has a neighbour
                uint4 q[U];
                float wq[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    q[u] = gather16<T, NARROW>(a, __shfl(idx, t + u * NB + g), row_bytes, lane_off);
                    if constexpr (VALS) wq[u] = __shfl(wgt, t + u * NB + g);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if constexpr (VALS) sum.add_scaled(q[u], wq[u]);
                    else sum.add(q[u]);
                }
            }
            if (t < cnt) {   // lanes past the end hold `none`
                const int live = (cnt - t + NB - 1) / NB;
                uint4 q[U];
                float wq[U];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (u < live) {
                        q[u] = gather16<T, NARROW>(a, __shfl(idx, t + u * NB + g), row_bytes, lane_off);
                        if constexpr (VALS) wq[u] = __shfl(wgt, t + u * NB + g);
                    }
                if constexpr (VALS) sum.template add_batch_scaled<U>(q, wq, live);
                else sum.template add_batch<U>(q, live);
            }
            idx = idx_next;
            wgt = wgt_next;
        }
        float tot[V];
        sum.template total<LOG_G>(tot);
        if (g == 0 && active) {
            if (seg.slot < 0) {
                finish_vec<T>(a, seg.row, node, s, cc * V, tot);
            } else {
                float* p = a.partial + (int64_t)seg.slot * a.F + cc * V;
#pragma unroll
                for (int v = 0; v < V; v += 4) {
                    const f32x4 o = {tot[v], tot[v + 1], tot[v + 2], tot[v + 3]};
                    if (a.stream_out) __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(p + v));
                    else *reinterpret_cast<f32x4*>(p + v) = o;
                }
            }
        }
    }
}

// NB = 64/G short rows side by side, lane group g on row g: no sum across lanes is needed and
// every per-row step (bounds, scale, store) is paid once per NB rows.  Each lane group fetches G
// of its row's column indices per load (one per lane) and hands them round with cross-lane
// moves; groups whose row has ended gather the zero row (kFirst, whose table has none: their row's
// first neighbour again, with weight 0).  `beg`, `len`, `zrow`, `node`, `s` are per-lane values, equal
// within a lane group; len < 0 for a group without a row (an empty row, len = 0, still gets its
// all-zero result stored).
template <typename T, int LOG_G, bool NARROW, int MODE>
__device__ __forceinline__ void run_short_rows(const LayerArgs<T>& a, const int32_t beg, const int32_t len,
                                               const int32_t zrow, const int32_t node, const float s,
                                               const int32_t idx_first, const float wgt_first, const int lane) {
    constexpr int G = 1 << LOG_G;
    constexpr int V = T::kVec;
    constexpr int U = kInFlight < G ? kInFlight : G;
    constexpr bool VALS = MODE != kPlain;
    const int c = lane & (G - 1);
    const int group_base = lane & ~(G - 1);
    const int chunks = a.F / V;
    const uint32_t row_bytes = (uint32_t)a.ld_in * (uint32_t)sizeof(typename T::elem);
    int32_t none = a.n;
    if constexpr (MODE == kFirst) {   // lane 0 of the group holds the row's first neighbour (row 0 for an empty row)
        none = __shfl(idx_first, group_base);
        if (len <= 0) none = 0;
    }
    const int32_t idx_start = (MODE == kFirst && c >= len) ? none : idx_first;
    int maxlen = len;  // longest row of the batch (wave-uniform)
#pragma unroll
    for (int off = G; off < 64; off <<= 1) {
        const int o = __shfl_xor(maxlen, off);
        maxlen = o > maxlen ? o : maxlen;
    }
    maxlen = __builtin_amdgcn_readfirstlane(maxlen);

    for (int cb = 0; cb < chunks; cb += G) {
        const int cc = cb + c;
        const bool active = cc < chunks;
        const uint32_t lane_off = active ? (uint32_t)cc * 16u : 0u;
        Sum<T> sum;
        sum.clear();
        int32_t idx = idx_start;
        float wgt = wgt_first;
        for (int base = 0; base < maxlen; base += G) {
            int32_t idx_next = none;
            float wgt_next = 0.0f;
            if (base + G + c < len) {
                idx_next = *(a.cols + beg + base + G + c);
                if constexpr (VALS) wgt_next = *(a.vals + beg + base + G + c);
            }
            const int steps = maxlen - base < G ? maxlen - base : G;
            for (int t = 0; t < steps; t += U) {
                const int live = steps - t < U ? steps - t : U;
                uint4 q[U];
                float wq[U];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (u < live) {
                        q[u] = gather16<T, NARROW>(a, __shfl(idx, group_base + t + u), row_bytes, lane_off);
                        if constexpr (VALS) wq[u] = __shfl(wgt, group_base + t + u);
                    }
                if constexpr (VALS) sum.template add_batch_scaled<U>(q, wq, live);
                else sum.template add_batch<U>(q, live);
            }
            idx = idx_next;
            wgt = wgt_next;
        }
        if constexpr (MODE == kFirst)
            if (len == 0) sum.clear();   // an empty row gathered row 0 with weight 0: its sum is 0 whatever row 0 holds
        if (active && len >= 0) finish_vec<T>(a, zrow, node, s, cc * V, sum.acc);
    }
}

constexpr int kWaves = 4;          // wavefronts per workgroup
constexpr int kShortPerWave = 8;   // short rows a wavefront works through, 64/G at a time
constexpr int kSingleBlocksPerXcd = 512;  // B-workgroups per XCD (fewer when the graph cannot have that many such rows)

// Three kinds of workgroup.
// A. Segments of rows cut into several (the first n_slot entries of the ordered segment list,
//    ordered by first column), one per wavefront.  The schedule deals the list out to the XCDs in
//    contiguous stretches of equal entry counts; the A-workgroups of XCD x take the segments of
//    stretch x in order, so the segments in flight on an XCD are consecutive ones, read the same
//    window of feature rows, and share it in that XCD's L2.  The launch is sized so that each
//    wavefront takes one segment, which keeps the segments in flight on an XCD next to each other in
//    the list (a stretch longer than the launch was sized for goes round again).  (Measured on the 50 M-edge
//    graph: with the A-workgroups capped at 2048 per XCD and going round their stretch three times,
//    three distant stretches of windows were in flight at once and the kernel fetched 12.0 GB per
//    launch instead of 10.7; the empty workgroups of the uncapped launch leave at once and cost
//    nothing measurable.)
// B. Rows of one segment, in row order; a fixed number of workgroups with equal shares.
// C. Short rows, kShortPerWave consecutive entries of the ordered short-row list per wavefront.
//    The wavefront fetches row numbers, bounds, node ids and scales of all its rows up front
//    (lane i holds row i's) and requests the next batch's first column indices before it works on
//    the current batch, so that no chain of dependent loads sits between batches.
// Workgroup b runs on XCD b mod 8 and XCDs take their workgroups in index order: on each XCD
// the sequence is its A-workgroups, then its share of B, then of C.  How many workgroups of each
// kind there really are is read from the schedule; the launch is sized for upper bounds and the
// workgroups beyond the real ones, all at the end of each XCD's sequence, leave at once.
// (Measured: spreading the L2-bound A-workgroups evenly among the HBM-bound others, so that both
// resources are busy all the time, was slower than running them one after the other.)
// At least four wavefronts per SIMD (128 registers): the instantiations that carry a value per entry
// would otherwise take 144 at 128-byte bf16 rows and lose a resident wavefront; none of them spills at 128.
template <typename T, int LOG_G, bool NARROW, int MODE>
__global__ __launch_bounds__(64 * kWaves) __attribute__((amdgpu_waves_per_eu(4))) void spmm_rows(const LayerArgs<T> a) {
    constexpr int G = 1 << LOG_G;
    constexpr int NB = 64 >> LOG_G;
    constexpr bool VALS = MODE != kPlain;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // The launch has one workgroup more than the schedule needs; it writes the all-zero row of the Z
    // buffer this layer fills and leaves.  (A workgroup of its own, so that no path of the others has
    // a store before its reads of the schedule: those then stay scalar loads.)
    if (blockIdx.x == gridDim.x - 1) {
        if (a.out_z) {
            const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
            for (int ch = threadIdx.x; ch < a.F / T::kVec; ch += 64 * kWaves)
                *reinterpret_cast<uint4*>(a.out_z + (int64_t)a.n * a.F + ch * T::kVec) = zero;
        }
        return;
    }
    const SchedHeader* h = a.sched.header;
    const bool refuse = refused<T>(a);
    const int x = blockIdx.x % kXcds;
    const int64_t j = blockIdx.x / kXcds;   // position in this XCD's sequence
    const int64_t a_lo = h->xcd_first[x], a_hi = h->xcd_first[x + 1];
    int64_t n_a = (a_hi - a_lo + kWaves - 1) / kWaves;
    if (n_a > a.a_blocks) n_a = a.a_blocks;   // a longer stretch than the launch was sized for: go round again
    const int64_t c_total = ((int64_t)h->n_short + kWaves * kShortPerWave - 1) / (kWaves * kShortPerWave);
    const int64_t n_b = a.b_blocks;                      // a fixed number, with equal shares of the rows
    const int64_t n_c = (c_total + kXcds - 1 - x) / kXcds;
    const int64_t total = n_a + n_b + n_c;
    if (j >= total) return;
    if (j < n_a) {
#pragma unroll 1
        for (int64_t t = a_lo + j * kWaves + wave; t < a_hi; t += n_a * kWaves)
            run_segment<T, LOG_G, NARROW, MODE>(a, a.sched.segs[t], lane, refuse);
        return;
    }
    const int64_t o = j - n_a;                           // position among the B- and C-workgroups
    if (o < n_b) {
        const int64_t lo = h->n_slot, hi = h->n_seg;
        const int64_t waves = n_b * kXcds * kWaves;
        const int64_t per_wave = (hi - lo + waves - 1) / waves;
        const int64_t first = lo + ((o * kXcds + x) * kWaves + wave) * per_wave;
        const int64_t last = first + per_wave < hi ? first + per_wave : hi;
#pragma unroll 1
        for (int64_t t = first; t < last; ++t) run_segment<T, LOG_G, NARROW, MODE>(a, a.sched.segs[t], lane, refuse);
        return;
    }
    const int64_t rb = (o - n_b) * kXcds + x;
    const int64_t n_short = a.sched.header->n_short;
    const int64_t first = ((int64_t)rb * kWaves + wave) * kShortPerWave;
    if (first >= n_short) return;
    const int n_rows = n_short - first < kShortPerWave ? (int)(n_short - first) : kShortPerWave;
    int32_t my_row = 0, my_beg = 0, my_len = -1, my_node = 0;
    float my_s = 0.0f;
    if (lane < n_rows) {
        my_row = a.sched.short_rows[first + lane];
        my_beg = a.sched.zrow_ptr[my_row];
        my_len = a.sched.zrow_ptr[my_row + 1] - my_beg;
        my_node = a.sched.orig[my_row];
        my_s = row_scale<T>(a, my_node, refuse);
    }
    const int c = lane & (G - 1);
    const int g = lane >> LOG_G;
    const int32_t none = MODE == kFirst ? 0 : a.n;
    int32_t beg = __shfl(my_beg, g), len = __shfl(my_len, g);
    int32_t idx_cur = c < len ? *(a.cols + beg + c) : none;
    float wgt_cur = 0.0f;
    if constexpr (VALS)
        if (c < len) wgt_cur = *(a.vals + beg + c);
#pragma unroll 1
    for (int r0 = 0; r0 < n_rows; r0 += NB) {
        const int src = r0 + g;      // the row of this lane's group (lanes >= n_rows hold len -1)
        const int nxt = (src + NB) & 63;
        const int32_t nbeg = __shfl(my_beg, nxt);
        const int32_t nlen = r0 + NB < n_rows ? __shfl(my_len, nxt) : -1;
        const int32_t idx_nxt = c < nlen ? *(a.cols + nbeg + c) : none;
        float wgt_nxt = 0.0f;
        if constexpr (VALS)
            if (c < nlen) wgt_nxt = *(a.vals + nbeg + c);
        run_short_rows<T, LOG_G, NARROW, MODE>(a, beg, len, __shfl(my_row, src), __shfl(my_node, src),
                                                   __shfl(my_s, src), idx_cur, wgt_cur, lane);
        beg = nbeg;
        len = nlen;
        idx_cur = idx_nxt;
        wgt_cur = wgt_nxt;
    }
}

constexpr int kReduceThreads = 256;
constexpr int kReduceBlocks = 8192;   // at most this many workgroups; they stride over the split rows

// Rows cut into segments: add their partial sums in a fixed order.  One workgroup per long row
// (the launch is sized for an upper bound of such rows that depends on nnz only, capped, and
// the workgroups stride over the real ones); thread (sl, cv) sums slots sl, sl+SL, ... of column
// quad cv in double, then the SL lane sums are added in lane order.
template <typename T>
__global__ __launch_bounds__(kReduceThreads) void reduce_split_rows(const LayerArgs<T> a) {
    constexpr int kThreads = kReduceThreads;
    __shared__ double red[kThreads][4];
    const int32_t n_multi = a.sched.header->n_multi;
    const bool refuse = refused<T>(a);
    for (int32_t m = blockIdx.x; m < n_multi; m += gridDim.x) {
    const int32_t k = a.sched.multi_row[m];  // internal row
    const int32_t node = a.sched.orig[k];
    const int32_t base = a.sched.slot_base[m];
    const int32_t cnt = a.sched.slot_cnt[m];
    const float s = row_scale<T>(a, node, refuse);
    const int quads = a.F / 4;
    for (int q0 = 0; q0 < quads; q0 += kThreads) {
        const int width = quads - q0 < kThreads ? quads - q0 : kThreads;
        const int lanes = kThreads / width;          // slot lanes
        const int sl = threadIdx.x / width;
        const int cv = threadIdx.x - sl * width;
        double sum[4] = {0.0, 0.0, 0.0, 0.0};
        if (sl < lanes) {
            const float* p = a.partial + (int64_t)base * a.F + (int64_t)(q0 + cv) * 4;
            // slots sl, sl + lanes, ... in that order; unrolled so that eight loads are in flight
#pragma unroll 8
            for (int32_t q = sl; q < cnt; q += lanes) {
                const float4 v0 = *reinterpret_cast<const float4*>(p + (int64_t)q * a.F);
                sum[0] += (double)v0.x; sum[1] += (double)v0.y; sum[2] += (double)v0.z; sum[3] += (double)v0.w;
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) red[threadIdx.x][e] = sum[e];
        __syncthreads();
        if (sl == 0) {
            for (int l = 1; l < lanes; ++l) {
#pragma unroll
                for (int e = 0; e < 4; ++e) sum[e] += red[l * width + cv][e];
            }
            const int col = (q0 + cv) * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float h = s * (float)sum[e];
                if (a.addend) h += load_one<T>(a.addend + (int64_t)node * a.ld_add + col + e);
                if (a.out_h) store_one<T>(a.out_h + (int64_t)node * a.ld_h + col + e, h);
                if (a.out_z) store_one<T>(a.out_z + (int64_t)k * a.F + col + e, s * h);
            }
        }
        __syncthreads();
    }
    }
}

constexpr int kPrescaleThreads = 256;

constexpr int64_t kDirectMaxNnz = 1 << 20;   // see run_layers
constexpr int kPrescaleRows = 4;   // rows per thread: their dependent loads (row -> node -> x, s) overlap

// Z = S_in X in internal row order: one streaming pass, 16 bytes of kPrescaleRows rows per thread.
// Also clears the zero row (index n) of the Z buffer (of both, if z_other is given).  Used for Z(0) of a
// multi-layer propagation (see run_layers) and by e2eg_aggregate, whose input scales depend on the mode.
template <typename T>
__global__ __launch_bounds__(kPrescaleThreads) void prescale_rows(const typename T::elem* __restrict__ x,
                                                                   int64_t ldx,
                                                                   const float* __restrict__ dinv_sqrt,
                                                                   const int32_t* __restrict__ orig,
                                                                   typename T::elem* __restrict__ z,
                                                                   typename T::elem* __restrict__ z_other,
                                                                   int64_t n, int32_t F, bool stream) {
    constexpr int V = T::kVec;
    const int chunks = F / V;
    const int64_t id = (int64_t)blockIdx.x * kPrescaleThreads + threadIdx.x;
    const int64_t groups = (n + 1 + kPrescaleRows - 1) / kPrescaleRows;
    if (id >= groups * chunks) return;
    const int64_t group = id / chunks;
    const int col = (int)(id - group * chunks) * V;
    int64_t node[kPrescaleRows];
#pragma unroll
    for (int i = 0; i < kPrescaleRows; ++i) {
        const int64_t zrow = group * kPrescaleRows + i;
        node[i] = zrow < n ? orig[zrow] : -1;
    }
    float v[kPrescaleRows][V];
    float s[kPrescaleRows];
#pragma unroll
    for (int i = 0; i < kPrescaleRows; ++i) {
        s[i] = 0.0f;
#pragma unroll
        for (int k = 0; k < V; ++k) v[i][k] = 0.0f;
        if (node[i] >= 0) {
            load_vec<T>(x + node[i] * ldx + col, v[i]);
            s[i] = dinv_sqrt[node[i]];
        }
    }
#pragma unroll
    for (int i = 0; i < kPrescaleRows; ++i) {
        const int64_t zrow = group * kPrescaleRows + i;
        if (zrow > n) continue;
#pragma unroll
        for (int k = 0; k < V; ++k) v[i][k] *= s[i];   // the zero row: 0 * 0
        store_vec<T>(z + zrow * F + col, v[i], stream);
        if (zrow == n && z_other) store_vec<T>(z_other + zrow * F + col, v[i], stream);
    }
}

template <typename T, bool NARROW, int MODE>
void launch_spmm(int log_g, dim3 grid, const LayerArgs<T>& a, hipStream_t stream) {
    const dim3 blk(64 * kWaves);
    switch (log_g) {
        case 0: spmm_rows<T, 0, NARROW, MODE><<<grid, blk, 0, stream>>>(a); break;
        case 1: spmm_rows<T, 1, NARROW, MODE><<<grid, blk, 0, stream>>>(a); break;
        case 2: spmm_rows<T, 2, NARROW, MODE><<<grid, blk, 0, stream>>>(a); break;
        case 3: spmm_rows<T, 3, NARROW, MODE><<<grid, blk, 0, stream>>>(a); break;
        case 4: spmm_rows<T, 4, NARROW, MODE><<<grid, blk, 0, stream>>>(a); break;
        case 5: spmm_rows<T, 5, NARROW, MODE><<<grid, blk, 0, stream>>>(a); break;
        default: spmm_rows<T, 6, NARROW, MODE><<<grid, blk, 0, stream>>>(a); break;
    }
}

// Results are streamed past the caches when one feature table is larger than this (see store_vec).
constexpr uint64_t kStreamOutBytes = 64ull << 20;
inline bool streams_out(uint64_t table_bytes) { return table_bytes > kStreamOutBytes; }

// `mode`: kPlain / kValues for a layer that reads a Z buffer (a.cols = zcol, a.vals = null / zval),
// kFirst for one that reads the caller's rows (a.cols = znode, a.vals = zs, a.ld_in = their leading dimension).
template <typename T>
int32_t launch_layer(LayerArgs<T>& a, int mode, int64_t n, int64_t nnz, hipStream_t stream) {
    const int chunks = a.F / T::kVec;
    int log_g = 0;
    while ((1 << log_g) < chunks && log_g < 6) ++log_g;
    const uint64_t row_bytes = (uint64_t)a.ld_in * sizeof(typename T::elem);
    const uint64_t table_bytes = (uint64_t)(n + 1) * row_bytes;
    // 32-bit byte offsets formed by a 24-bit multiply: both factors below 2^24, the table below 4 GiB
    const bool narrow = table_bytes <= 0xffffffffull && n + 1 <= (1 << 24) && row_bytes < (1u << 24);
    // upper bounds of the three kinds of workgroup (see spmm_rows), per XCD, times the XCDs.  The bound
    // on slotted segments is about three times what a graph really has, so an eighth of it per XCD
    // covers every stretch the deal by entry counts produces in practice; a longer one goes round again.
    int64_t a_blocks = nnz > kSegLen ? ceil_div(ceil_div(sched_max_slot(n, nnz), kWaves), kXcds) + 1 : 0;
    int64_t b_blocks = nnz > kShortMax ? ceil_div(ceil_div(sched_max_plain(nnz), kWaves), kXcds) + 1 : 0;
    if (b_blocks > kSingleBlocksPerXcd) b_blocks = kSingleBlocksPerXcd;
    const int64_t c_blocks = ceil_div(ceil_div(n, kWaves * kShortPerWave), kXcds) + 1;
    a.n = (int32_t)n;
    a.stream_out = streams_out((uint64_t)(n + 1) * (uint64_t)a.F * sizeof(typename T::elem)) ? 1 : 0;
    a.a_blocks = (int32_t)a_blocks;
    a.b_blocks = (int32_t)b_blocks;
    const dim3 grid((unsigned)(kXcds * (a_blocks + b_blocks + c_blocks) + 1));   // the last one: see spmm_rows
    profile_mark(stream, false);
    if (mode == kFirst) {
        if (narrow) launch_spmm<T, true, kFirst>(log_g, grid, a, stream);
        else launch_spmm<T, false, kFirst>(log_g, grid, a, stream);
    } else if (mode == kValues) {
        if (narrow) launch_spmm<T, true, kValues>(log_g, grid, a, stream);
        else launch_spmm<T, false, kValues>(log_g, grid, a, stream);
    } else {
        if (narrow) launch_spmm<T, true, kPlain>(log_g, grid, a, stream);
        else launch_spmm<T, false, kPlain>(log_g, grid, a, stream);
    }
    profile_mark(stream, true);
    E2EG_LAUNCH_CHECK("spmm_rows");
    if (nnz > kSegLen) {  // otherwise no row has several segments
        const int64_t blocks = sched_max_multi(nnz) < kReduceBlocks ? sched_max_multi(nnz) : kReduceBlocks;
        reduce_split_rows<T><<<dim3((unsigned)blocks), dim3(kReduceThreads), 0, stream>>>(a);
        E2EG_LAUNCH_CHECK("reduce_split_rows");
    }
    return E2EG_OK;
}

struct PropWs {
    void* z[2];
    float* partial;
    size_t bytes;
};

PropWs carve_prop(void* base, int64_t n, int64_t nnz, int32_t dtype, int32_t F, int32_t K) {
    Carver c(base);
    PropWs w;
    const size_t esz = dtype == E2EG_F32 ? 4 : 2;
    const size_t zbytes = (size_t)(n + 1) * (size_t)F * esz;  // one extra all-zero row
    w.z[0] = c.take<char>(zbytes);
    w.z[1] = K > 1 ? c.take<char>(zbytes) : nullptr;
    w.partial = c.take<float>((size_t)sched_max_slot(n, nnz) * (size_t)F);
    w.bytes = c.size();
    return w;
}

int32_t check_common(const char* who, int32_t n, int64_t nnz, const void* row_ptr, const void* col_idx,
                     const void* dinv, const void* sched, int32_t dtype, int32_t F, int32_t K) {
    if (n < 0 || nnz < 0) return fail(E2EG_ERR_INVALID_ARG, "%s: negative size", who);
    if (nnz > (int64_t)INT32_MAX || n == INT32_MAX)
        return fail(E2EG_ERR_OVERFLOW, "%s: nnz=%lld exceeds int32", who, (long long)nnz);
    if (dtype != E2EG_F32 && dtype != E2EG_BF16) return fail(E2EG_ERR_BAD_DTYPE, "%s: dtype %d", who, dtype);
    const int vec = dtype == E2EG_F32 ? 4 : 8;
    if (F <= 0 || F % vec != 0)
        return fail(E2EG_ERR_INVALID_ARG, "%s: F=%d must be a positive multiple of %d", who, F, vec);
    if (K < 1) return fail(E2EG_ERR_INVALID_ARG, "%s: K=%d must be >= 1", who, K);
    if (!row_ptr || !dinv || !sched || (nnz > 0 && !col_idx))
        return fail(E2EG_ERR_NULL_PTR, "%s: null graph pointer", who);
    return E2EG_OK;
}

int32_t check_matrix(const char* who, const char* name, const void* p, int64_t ld, int32_t F, int32_t dtype) {
    const int vec = dtype == E2EG_F32 ? 4 : 8;
    if (!p) return fail(E2EG_ERR_NULL_PTR, "%s: %s is null", who, name);
    if (!aligned_to(p, 16)) return fail(E2EG_ERR_INVALID_ARG, "%s: %s is not 16-byte aligned", who, name);
    if (ld < F || ld % vec != 0)
        return fail(E2EG_ERR_INVALID_ARG, "%s: leading dimension of %s (%lld) must be >= F and a multiple of %d",
                    who, name, (long long)ld, vec);
    return E2EG_OK;
}

// Runs K layers.  `in` is the layer-K-side input (X0 for forward, dL/dH(K) for backward);
// outputs: layer index L = 1..K in forward order.  store(L) says where H of the L-th computed
// layer goes (null = not kept); add(L) is the direct term added to it (null = none).
template <typename T>
int32_t run_layers(int32_t n, int64_t nnz, const int32_t* row_ptr, const int32_t* col_idx,
                   const float* dinv, const void* sched, int32_t F, int32_t K, const void* in,
                   int64_t ld_in, typename T::elem* const* store, const int64_t* ld_store,
                   const typename T::elem* const* add, int64_t ld_add, const PropWs& w,
                   bool weighted, bool transposed, hipStream_t stream) {
    using E = typename T::elem;
    SchedView view;
    sched_carve(const_cast<void*>(sched), n, nnz, &view, weighted);
    // Layer l > 1 reads Z(l-1), which layer l-1 wrote into one of the two Z buffers (each launch also
    // writes the all-zero row of the buffer it fills).  Layer 1 reads either Z(0), made by a streaming
    // pre-scale pass, or the caller's rows themselves (kFirst).  The direct form saves that pass
    // (2 n row-bytes, a launch, a rounding) and pays for it with a value per entry to read, hand round
    // and multiply by (4 nnz bytes more).  It is taken when that trade is good: 4 nnz < 2 n row-bytes,
    // or a graph so small (kDirectMaxNnz entries) that a launch costs as much as the layer.  Measured
    // (ms per K = 3 forward, pre-scale / direct): 2 M edges, 256-byte rows 0.63 / 0.62; 50 M edges,
    // 256-byte rows 5.78 / 5.67; 50 M edges, 128-byte rows 7.37 / 7.53 - the one the rule sends the
    // other way.
    const uint64_t row_bytes_in = (uint64_t)F * sizeof(E);
    const bool direct = nnz <= kDirectMaxNnz || 2 * (uint64_t)nnz < (uint64_t)n * row_bytes_in;
    E* z_bufs[2] = {static_cast<E*>(w.z[0]), static_cast<E*>(w.z[1])};
    int cur = -1;   // the Z buffer the next layer reads; -1: the caller's rows
    if (!direct) {
        const int chunks = F / T::kVec;
        prescale_rows<T><<<dim3((unsigned)ceil_div(ceil_div((int64_t)n + 1, kPrescaleRows) * chunks, kPrescaleThreads)),
                           dim3(kPrescaleThreads), 0, stream>>>(static_cast<const E*>(in), ld_in, dinv, view.orig,
                                                                z_bufs[0], nullptr, n, F,
                                                                streams_out((uint64_t)(n + 1) * F * sizeof(E)));
        E2EG_LAUNCH_CHECK("prescale_rows");
        cur = 0;
    }
    for (int32_t l = 1; l <= K; ++l) {
        LayerArgs<T> a;
        a.dinv_sqrt = dinv;
        a.sched = view;
        a.transposed = transposed ? 1 : 0;
        int mode;
        if (cur < 0) {
            a.zin = static_cast<const E*>(in);
            a.ld_in = ld_in;
            a.cols = view.znode;
            a.vals = view.zs;
            mode = kFirst;
        } else {
            a.zin = z_bufs[cur];
            a.ld_in = F;
            a.cols = view.zcol;
            a.vals = weighted ? view.zval : nullptr;
            mode = weighted ? kValues : kPlain;
        }
        const int nxt = cur < 0 ? 0 : 1 - cur;
        a.out_h = store[l - 1];
        a.ld_h = ld_store[l - 1];
        a.out_z = l < K ? z_bufs[nxt] : nullptr;
        a.addend = add ? add[l - 1] : nullptr;
        a.ld_add = ld_add;
        a.partial = w.partial;
        a.F = F;
        int32_t st = launch_layer<T>(a, mode, n, nnz, stream);
        if (st != E2EG_OK) return st;
        cur = nxt;
    }
    return E2EG_OK;
}

// Per-node input and output scales of e2eg_aggregate, from the row lengths of the caller's CSR.
__global__ void aggregate_scales(const int32_t* __restrict__ row_ptr, int64_t n, int32_t mode,
                                 float* __restrict__ scale_in, float* __restrict__ scale_out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t d = row_ptr[i + 1] - row_ptr[i];
    const float inv = d > 0 ? (float)(1.0 / (double)d) : 0.0f;
    const float rs = d > 0 ? (float)(1.0 / sqrt((double)d)) : 0.0f;
    float in = 1.0f, out = 1.0f;
    if (mode == E2EG_AGG_SYM) in = out = rs;
    else if (mode == E2EG_AGG_MEAN) out = inv;
    else if (mode == E2EG_AGG_MEAN_T) in = inv;
    scale_in[i] = in;
    scale_out[i] = out;
}

struct AggWs {
    void* z;
    float* partial;
    float* scale_in;
    float* scale_out;
    size_t bytes;
};

AggWs carve_agg(void* base, int64_t n, int64_t nnz, int32_t dtype, int32_t F) {
    Carver c(base);
    AggWs w;
    const size_t esz = dtype == E2EG_F32 ? 4 : 2;
    w.z = c.take<char>((size_t)(n + 1) * (size_t)F * esz);
    w.partial = c.take<float>((size_t)sched_max_slot(n, nnz) * (size_t)F);
    w.scale_in = c.take<float>(n > 0 ? n : 1);
    w.scale_out = c.take<float>(n > 0 ? n : 1);
    w.bytes = c.size();
    return w;
}

template <typename T>
int32_t run_aggregate(int32_t mode, int32_t n, int64_t nnz, const int32_t* row_ptr, const void* sched, int32_t F,
                      const void* x, int64_t ldx, const void* addend, int64_t ld_add, void* y, int64_t ldy,
                      const AggWs& w, hipStream_t stream) {
    using E = typename T::elem;
    SchedView view;
    sched_carve(const_cast<void*>(sched), n, nnz, &view);
    aggregate_scales<<<dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, stream>>>(row_ptr, n, mode, w.scale_in,
                                                                                w.scale_out);
    E2EG_LAUNCH_CHECK("aggregate_scales");
    const int chunks = F / T::kVec;
    prescale_rows<T><<<dim3((unsigned)ceil_div(ceil_div((int64_t)n + 1, kPrescaleRows) * chunks, kPrescaleThreads)),
                       dim3(kPrescaleThreads), 0, stream>>>(static_cast<const E*>(x), ldx, w.scale_in, view.orig,
                                                            static_cast<E*>(w.z), nullptr, n, F,
                                                            streams_out((uint64_t)(n + 1) * F * sizeof(E)));
    E2EG_LAUNCH_CHECK("prescale_rows");
    LayerArgs<T> a;
    a.dinv_sqrt = w.scale_out;
    a.sched = view;
    a.zin = static_cast<const E*>(w.z);
    a.ld_in = F;
    a.cols = view.zcol;
    a.vals = nullptr;
    a.transposed = mode == E2EG_AGG_MEAN_T ? 1 : 0;
    a.out_h = static_cast<E*>(y);
    a.ld_h = ldy;
    a.out_z = nullptr;
    a.addend = static_cast<const E*>(addend);
    a.ld_add = ld_add;
    a.partial = w.partial;
    a.F = F;
    return launch_layer<T>(a, kPlain, n, nnz, stream);
}

constexpr int kMaxLayers = 64;

}  // namespace
}  // namespace e2eg

using namespace e2eg;

extern "C" size_t e2eg_propagate_workspace_bytes(int32_t n, int64_t nnz, int32_t dtype, int32_t F,
                                                 int32_t K) {
    if (n < 0 || nnz < 0 || F <= 0 || K < 1 || (dtype != E2EG_F32 && dtype != E2EG_BF16)) return 0;
    return carve_prop(nullptr, n, nnz, dtype, F, K).bytes;
}

namespace {
// `weighted` says which of the two schedule layouts d_sched holds (the weighted one carries the
// entries' values, which the kernel then multiplies in).
int32_t propagate_fwd_impl(bool weighted, int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                           const int32_t* d_col_idx, const float* d_dinv_sqrt, const void* d_sched,
                           int32_t dtype, int32_t F, int32_t K, const void* d_X0, int64_t ldx, void* d_Xout,
                           int64_t ldo, int64_t layer_stride, void* ws, size_t ws_bytes, void* stream_) {
    const char* who = weighted ? "propagate_weighted_fwd" : "propagate_fwd";
    int32_t st = check_common(who, n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, dtype, F, K);
    if (st != E2EG_OK) return st;
    if (K > kMaxLayers) return fail(E2EG_ERR_INVALID_ARG, "%s: K=%d exceeds %d", who, K, kMaxLayers);
    if ((st = check_matrix(who, "d_X0", d_X0, ldx, F, dtype)) != E2EG_OK) return st;
    if ((st = check_matrix(who, "d_Xout", d_Xout, ldo, F, dtype)) != E2EG_OK) return st;
    const int vec = dtype == E2EG_F32 ? 4 : 8;
    if (layer_stride != 0 && (layer_stride < (int64_t)n * ldo || layer_stride % vec != 0))
        return fail(E2EG_ERR_INVALID_ARG, "%s: layer_stride %lld must be 0 or >= n*ldo and a multiple of %d",
                    who, (long long)layer_stride, vec);
    const size_t need = e2eg_propagate_workspace_bytes(n, nnz, dtype, F, K);
    if (!ws || !aligned_to(ws, kAlign) || ws_bytes < need)
        return fail(E2EG_ERR_WORKSPACE, "%s: workspace needs %zu bytes, 256-byte aligned", who, need);
    if (n == 0) return E2EG_OK;

    hipStream_t stream = static_cast<hipStream_t>(stream_);
    PropWs w = carve_prop(ws, n, nnz, dtype, F, K);
    int64_t lds[kMaxLayers];
    for (int l = 0; l < K; ++l) lds[l] = ldo;
    if (dtype == E2EG_F32) {
        float* store[kMaxLayers];
        for (int l = 1; l <= K; ++l)
            store[l - 1] = layer_stride ? static_cast<float*>(d_Xout) + (int64_t)(l - 1) * layer_stride
                                        : (l == K ? static_cast<float*>(d_Xout) : nullptr);
        return run_layers<F32>(n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, F, K, d_X0, ldx, store,
                               lds, nullptr, 0, w, weighted, false, stream);
    }
    uint16_t* store[kMaxLayers];
    for (int l = 1; l <= K; ++l)
        store[l - 1] = layer_stride ? static_cast<uint16_t*>(d_Xout) + (int64_t)(l - 1) * layer_stride
                                    : (l == K ? static_cast<uint16_t*>(d_Xout) : nullptr);
    return run_layers<BF16>(n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, F, K, d_X0, ldx, store,
                            lds, nullptr, 0, w, weighted, false, stream);
}

int32_t propagate_bwd_impl(bool weighted, int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                           const int32_t* d_col_idx, const float* d_dinv_sqrt, const void* d_sched,
                           int32_t dtype, int32_t F, int32_t K, const void* d_gXK, int64_t ldg,
                           const void* d_gLayers, int64_t g_layer_stride, void* d_gX0, int64_t ldo, void* ws,
                           size_t ws_bytes, void* stream_) {
    const char* who = weighted ? "propagate_weighted_bwd" : "propagate_bwd";
    int32_t st = check_common(who, n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, dtype, F, K);
    if (st != E2EG_OK) return st;
    if (K > kMaxLayers) return fail(E2EG_ERR_INVALID_ARG, "%s: K=%d exceeds %d", who, K, kMaxLayers);
    if ((st = check_matrix(who, "d_gXK", d_gXK, ldg, F, dtype)) != E2EG_OK) return st;
    if ((st = check_matrix(who, "d_gX0", d_gX0, ldo, F, dtype)) != E2EG_OK) return st;
    const int vec = dtype == E2EG_F32 ? 4 : 8;
    const bool shared_term = d_gLayers && g_layer_stride == 0;  // one direct term for layers 0..K-1
    if (d_gLayers && (K > 1 || shared_term)) {
        if (!aligned_to(d_gLayers, 16)) return fail(E2EG_ERR_INVALID_ARG, "%s: d_gLayers is not 16-byte aligned", who);
        if (!shared_term && (g_layer_stride < (int64_t)n * ldg || g_layer_stride % vec != 0))
            return fail(E2EG_ERR_INVALID_ARG, "%s: g_layer_stride %lld must be 0 or >= n*ldg and a multiple of %d",
                        who, (long long)g_layer_stride, vec);
    }
    const size_t need = e2eg_propagate_workspace_bytes(n, nnz, dtype, F, K);
    if (!ws || !aligned_to(ws, kAlign) || ws_bytes < need)
        return fail(E2EG_ERR_WORKSPACE, "%s: workspace needs %zu bytes, 256-byte aligned", who, need);
    if (n == 0) return E2EG_OK;

    hipStream_t stream = static_cast<hipStream_t>(stream_);
    PropWs w = carve_prop(ws, n, nnz, dtype, F, K);
    int64_t lds[kMaxLayers];
    for (int l = 0; l < K; ++l) lds[l] = ldo;
    // Computed layer L (1..K) is G(K-L); its direct term is D(K-L), given for 1 <= K-L <= K-1.
    if (dtype == E2EG_F32) {
        float* store[kMaxLayers];
        const float* add[kMaxLayers];
        for (int L = 1; L <= K; ++L) {
            const int l = K - L;
            store[L - 1] = L == K ? static_cast<float*>(d_gX0) : nullptr;
            add[L - 1] = shared_term ? static_cast<const float*>(d_gLayers)
                         : (d_gLayers && l >= 1) ? static_cast<const float*>(d_gLayers) + (int64_t)(l - 1) * g_layer_stride
                                                 : nullptr;
        }
        return run_layers<F32>(n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, F, K, d_gXK, ldg, store,
                               lds, add, ldg, w, weighted, true, stream);
    }
    uint16_t* store[kMaxLayers];
    const uint16_t* add[kMaxLayers];
    for (int L = 1; L <= K; ++L) {
        const int l = K - L;
        store[L - 1] = L == K ? static_cast<uint16_t*>(d_gX0) : nullptr;
        add[L - 1] = shared_term ? static_cast<const uint16_t*>(d_gLayers)
                     : (d_gLayers && l >= 1) ? static_cast<const uint16_t*>(d_gLayers) + (int64_t)(l - 1) * g_layer_stride
                                             : nullptr;
    }
    return run_layers<BF16>(n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, F, K, d_gXK, ldg, store,
                            lds, add, ldg, w, weighted, true, stream);
}
}  // namespace

extern "C" int32_t e2eg_propagate_fwd(int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                                      const int32_t* d_col_idx, const float* d_dinv_sqrt,
                                      const void* d_sched, int32_t dtype, int32_t F, int32_t K,
                                      const void* d_X0, int64_t ldx, void* d_Xout, int64_t ldo,
                                      int64_t layer_stride, void* ws, size_t ws_bytes, void* stream) {
    return propagate_fwd_impl(false, n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, dtype, F, K, d_X0, ldx,
                              d_Xout, ldo, layer_stride, ws, ws_bytes, stream);
}

extern "C" int32_t e2eg_propagate_weighted_fwd(int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                                               const int32_t* d_col_idx, const float* d_dinv_sqrt,
                                               const void* d_sched, int32_t dtype, int32_t F, int32_t K,
                                               const void* d_X0, int64_t ldx, void* d_Xout, int64_t ldo,
                                               int64_t layer_stride, void* ws, size_t ws_bytes, void* stream) {
    return propagate_fwd_impl(true, n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, dtype, F, K, d_X0, ldx,
                              d_Xout, ldo, layer_stride, ws, ws_bytes, stream);
}

extern "C" int32_t e2eg_propagate_bwd(int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                                      const int32_t* d_col_idx, const float* d_dinv_sqrt,
                                      const void* d_sched, int32_t dtype, int32_t F, int32_t K,
                                      const void* d_gXK, int64_t ldg, const void* d_gLayers,
                                      int64_t g_layer_stride, void* d_gX0, int64_t ldo, void* ws,
                                      size_t ws_bytes, void* stream) {
    return propagate_bwd_impl(false, n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, dtype, F, K, d_gXK, ldg,
                              d_gLayers, g_layer_stride, d_gX0, ldo, ws, ws_bytes, stream);
}

extern "C" int32_t e2eg_propagate_weighted_bwd(int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                                               const int32_t* d_col_idx, const float* d_dinv_sqrt,
                                               const void* d_sched, int32_t dtype, int32_t F, int32_t K,
                                               const void* d_gXK, int64_t ldg, const void* d_gLayers,
                                               int64_t g_layer_stride, void* d_gX0, int64_t ldo, void* ws,
                                               size_t ws_bytes, void* stream) {
    return propagate_bwd_impl(true, n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, dtype, F, K, d_gXK, ldg,
                              d_gLayers, g_layer_stride, d_gX0, ldo, ws, ws_bytes, stream);
}

extern "C" size_t e2eg_aggregate_workspace_bytes(int32_t n, int64_t nnz, int32_t dtype, int32_t F) {
    if (n < 0 || nnz < 0 || F <= 0 || (dtype != E2EG_F32 && dtype != E2EG_BF16)) return 0;
    return carve_agg(nullptr, n, nnz, dtype, F).bytes;
}

extern "C" int32_t e2eg_aggregate(int32_t mode, int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                                  const int32_t* d_col_idx, const void* d_sched, int32_t dtype, int32_t F,
                                  const void* d_X, int64_t ldx, const void* d_addend, int64_t ld_add, void* d_Y,
                                  int64_t ldy, void* ws, size_t ws_bytes, void* stream_) {
    const char* who = "aggregate";
    if (mode != E2EG_AGG_SYM && mode != E2EG_AGG_MEAN && mode != E2EG_AGG_MEAN_T && mode != E2EG_AGG_SUM)
        return fail(E2EG_ERR_INVALID_ARG, "%s: mode %d", who, mode);
    const float one = 1.0f;  // stands for the scale array in the shared checks; never dereferenced
    int32_t st = check_common(who, n, nnz, d_row_ptr, d_col_idx, &one, d_sched, dtype, F, 1);
    if (st != E2EG_OK) return st;
    if ((st = check_matrix(who, "d_X", d_X, ldx, F, dtype)) != E2EG_OK) return st;
    if ((st = check_matrix(who, "d_Y", d_Y, ldy, F, dtype)) != E2EG_OK) return st;
    if (d_addend && (st = check_matrix(who, "d_addend", d_addend, ld_add, F, dtype)) != E2EG_OK) return st;
    const size_t need = e2eg_aggregate_workspace_bytes(n, nnz, dtype, F);
    if (!ws || !aligned_to(ws, kAlign) || ws_bytes < need)
        return fail(E2EG_ERR_WORKSPACE, "%s: workspace needs %zu bytes, 256-byte aligned", who, need);
    if (n == 0) return E2EG_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const AggWs w = carve_agg(ws, n, nnz, dtype, F);
    if (dtype == E2EG_F32)
        return run_aggregate<F32>(mode, n, nnz, d_row_ptr, d_sched, F, d_X, ldx, d_addend, ld_add, d_Y, ldy, w, stream);
    return run_aggregate<BF16>(mode, n, nnz, d_row_ptr, d_sched, F, d_X, ldx, d_addend, ld_add, d_Y, ldy, w, stream);
}
