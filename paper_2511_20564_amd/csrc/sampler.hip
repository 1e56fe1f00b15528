// Importance sampling of a multi-hop subgraph (paper: Section 4.1, the sampling probability
// p(u->v) = w_uv^beta / sum_k w_uk^beta with at most k neighbours per node and depth L; Section 5,
// "Subgraph Sampling": fan-outs per hop).
//
// Design for the GPU: every decision is integer arithmetic, so the result is a function of the
// inputs and the seed alone.
//   * e2eg_sampler_prepare turns each row's weights into integers (2^24 at the row maximum, the
//     division decided in fp32 with IEEE rounding) and prefix-sums them over the whole CSR: the
//     table holds cum[e] = sum of the integer weights before entry e, nnz + 1 values of 64 bits.
//     One thread per entry throughout, so that a row of a million entries is no wavefront's loop.
//   * a draw is one thread: 64 random bits from the counter-based generator Philox4x32-10 (Salmon,
//     Moraes, Dror, Shaw, SC 2011; counter = (draw, node, hop, 0), key = the seed), scaled to the
//     row total by a 64x64->128-bit multiply, then a binary search in the row's slice of the table.
//   * visited nodes are marked with an integer compare-and-swap (all writers of one hop write the
//     same value); frontiers, the node list and the edge list are compacted with prefix sums, so
//     their order is ascending node id / draw order and does not depend on scheduling.
//   * launch sizes come from upper bounds (seeds x fan-outs); the real frontier sizes stay on the
//     device.  The one wait is at the end, for the three counts handed to the host.
#include "common.h"

namespace e2eg {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxHops = 8;
constexpr int kMaxFanout = 1 << 16;

inline dim3 grid_for(int64_t count) { return dim3((unsigned)ceil_div(count > 0 ? count : 1, kThreads)); }

__device__ __forceinline__ bool usable(float p) { return p > 0.0f && p <= 3.402823466e38f; }

__global__ void pow_weights(const float* __restrict__ val, int64_t nnz, float beta, float* __restrict__ p) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= nnz) return;
    const float v = val[e];
    float r = 0.0f;
    if (v > 0.0f) r = beta == 1.0f ? v : beta == 0.0f ? 1.0f : powf(v, beta);
    p[e] = r;
}

// The row of entry e: the last i in [lo, hi] with row_ptr[i] <= e.
__device__ __forceinline__ int64_t row_of_entry(const int32_t* __restrict__ row_ptr, int64_t e, int64_t lo, int64_t hi) {
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (row_ptr[mid] <= e) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Rows of a workgroup's (consecutive) entries: two threads search all rows for the first and the last
// entry's, every thread then searches that short range.  -> the row of entry `e` (e < nnz).
__device__ __forceinline__ int64_t row_in_block(const int32_t* __restrict__ row_ptr, int64_t n, int64_t nnz,
                                                int64_t first, int64_t e, int64_t* range) {
    if (threadIdx.x == 0) range[0] = row_of_entry(row_ptr, first, 0, n - 1);
    if (threadIdx.x == 64) {
        const int64_t last = first + kThreads - 1 < nnz ? first + kThreads - 1 : nnz - 1;
        range[1] = row_of_entry(row_ptr, last, 0, n - 1);
    }
    __syncthreads();
    return e < nnz ? row_of_entry(row_ptr, e, range[0], range[1]) : -1;
}

// One thread per entry: the largest usable weight off the diagonal of every row, as the bit pattern
// of a positive float (which orders like an integer).  The entries of a row are neighbours, so a
// wavefront first takes the maximum of each run of equal rows among its lanes and only the first
// lane of a run goes to memory: a row of a million entries costs some ten thousand atomics.
__global__ __launch_bounds__(kThreads) void row_max(const int32_t* __restrict__ row_ptr,
                                                    const int32_t* __restrict__ col_idx, const float* __restrict__ p,
                                                    int64_t n, int64_t nnz, int32_t* row_max_bits) {
    __shared__ int64_t range[2];
    const int64_t first = (int64_t)blockIdx.x * kThreads;
    const int64_t e = first + threadIdx.x;
    const int64_t row = row_in_block(row_ptr, n, nnz, first, e, range);
    const int lane = threadIdx.x & 63;
    int32_t bits = 0;
    if (row >= 0) {
        const float v = p[e];
        if (col_idx[e] != (int32_t)row && usable(v)) bits = __float_as_int(v);
    }
    const int32_t r32 = (int32_t)row;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int32_t other = __shfl_down(bits, d, 64);
        const int32_t other_row = __shfl_down(r32, d, 64);
        if (lane + d < 64 && other_row == r32 && other > bits) bits = other;
    }
    const int32_t before = __shfl_up(r32, 1, 64);
    if (row >= 0 && (lane == 0 || before != r32) && bits > 0) atomicMax(row_max_bits + row, bits);
}

// One thread per entry: its integer weight.  The entry past the end gets the 0 that closes the scan.
__global__ __launch_bounds__(kThreads) void quantise_entries(const int32_t* __restrict__ row_ptr,
                                                             const int32_t* __restrict__ col_idx,
                                                             const float* __restrict__ p, int64_t n, int64_t nnz,
                                                             const int32_t* __restrict__ row_max_bits,
                                                             uint64_t* __restrict__ q) {
    __shared__ int64_t range[2];
    const int64_t first = (int64_t)blockIdx.x * kThreads;
    const int64_t e = first + threadIdx.x;
    if (e == nnz) q[nnz] = 0;
    if (first >= nnz) return;   // the whole workgroup (only the one that holds entry nnz alone)
    const int64_t row = row_in_block(row_ptr, n, nnz, first, e, range);
    if (row < 0) return;
    const float v = p[e];
    uint64_t w = 0;
    if (col_idx[e] != (int32_t)row && usable(v)) {
        const float pmax = __int_as_float(row_max_bits[row]);
        const float scaled = floorf(__fmul_rn(__fdiv_rn(v, pmax), 16777216.0f));
        w = scaled >= 1.0f ? (uint64_t)scaled : 1u;
    }
    q[e] = w;
}

__global__ void fill_i32(int32_t* __restrict__ p, int64_t count, int32_t v) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = v;
}

__global__ void mark_seeds(const int32_t* __restrict__ seeds, int32_t n_seeds, int32_t n, int32_t* hop_of,
                           int32_t* __restrict__ bad) {
    const int32_t s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n_seeds) return;
    const int32_t v = seeds[s];
    if (v < 0 || v >= n) {
        atomicOr(bad, 1);
        return;
    }
    hop_of[v] = 1;
}

// flags[i] = 1 where hop_of[i] matches (`level` > 0: equal to it; `level` == 0: any visited node);
// flags[n] = 0 closes the scan.
__global__ void level_flags(const int32_t* __restrict__ hop_of, int32_t n, int32_t level, int32_t* __restrict__ flags) {
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n) return;
    int32_t f = 0;
    if (i < n) f = level > 0 ? (hop_of[i] == level) : (hop_of[i] > 0);
    flags[i] = f;
}

__global__ void scatter_level(const int32_t* __restrict__ hop_of, int32_t n, int32_t level,
                              const int32_t* __restrict__ pos, int32_t* __restrict__ out, int64_t capacity) {
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const bool hit = level > 0 ? (hop_of[i] == level) : (hop_of[i] > 0);
    if (hit && pos[i] < capacity) out[pos[i]] = i;
}

struct Philox {
    uint32_t c[4];
};

__device__ __forceinline__ Philox philox4x32_10(Philox x, uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, x.c[0]), lo0 = 0xD2511F53u * x.c[0];
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, x.c[2]), lo1 = 0xCD9E8D57u * x.c[2];
        Philox y;
        y.c[0] = hi1 ^ x.c[1] ^ k0;
        y.c[1] = lo1;
        y.c[2] = hi0 ^ x.c[3] ^ k1;
        y.c[3] = lo0;
        x = y;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return x;
}

// One thread per (frontier position f, draw t) of hop `hop`, for the upper bound `front_cap` of the
// frontier's size; the real size is *front_count.  Every slot of the hop is written: the source
// node, the picked neighbour (or -1: no pick) and the index of the stored entry.
__global__ void draw_picks(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                           const uint64_t* __restrict__ cum, const int32_t* __restrict__ frontier,
                           const int32_t* __restrict__ front_count, int64_t front_cap, int32_t k, int32_t hop,
                           uint32_t seed_lo, uint32_t seed_hi, int32_t* hop_of, int32_t* __restrict__ slot_src,
                           int32_t* __restrict__ slot_dst, int32_t* __restrict__ slot_ent) {
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= front_cap * k) return;
    const int64_t f = s / k;
    const int32_t t = (int32_t)(s - f * k);
    int32_t u = -1, v = -1, ent = -1;
    if (f < *front_count) {
        u = frontier[f];
        const int32_t beg = row_ptr[u], end = row_ptr[u + 1];
        // A node with at most k neighbours keeps every one that can be drawn at all.  Its row may
        // also hold the node itself (the diagonal entry, never drawn), so a row of k + 1 entries
        // qualifies when one of them is the diagonal: slot t then takes the t-th entry beside it.
        int32_t diag = -1;   // where the diagonal entry sits, looked for only where it decides
        if (end - beg == k + 1) {
            int32_t lo = beg, hi = end;   // first entry with column >= u (columns ascend)
            while (lo < hi) {
                const int32_t mid = lo + ((hi - lo) >> 1);
                if (col_idx[mid] < u) lo = mid + 1; else hi = mid;
            }
            if (lo < end && col_idx[lo] == u) diag = lo;
        }
        if (end - beg <= k) {
            if (t < end - beg && cum[beg + t + 1] > cum[beg + t]) ent = beg + t;
        } else if (diag >= 0) {
            const int32_t e = beg + t + (beg + t >= diag ? 1 : 0);
            if (cum[e + 1] > cum[e]) ent = e;
        } else {
            const uint64_t base = cum[beg], total = cum[end] - base;
            if (total > 0) {
                Philox x;
                x.c[0] = (uint32_t)t;
                x.c[1] = (uint32_t)u;
                x.c[2] = (uint32_t)hop;
                x.c[3] = 0u;
                x = philox4x32_10(x, seed_lo, seed_hi);
                const uint64_t bits = (uint64_t)x.c[0] | ((uint64_t)x.c[1] << 32);
                const uint64_t r = __umul64hi(bits, total);  // uniform on [0, total)
                int32_t lo = beg, hi = end - 1;              // smallest e with cum[e + 1] - base > r
                while (lo < hi) {
                    const int32_t mid = lo + ((hi - lo) >> 1);
                    if (cum[mid + 1] - base > r) hi = mid; else lo = mid + 1;
                }
                ent = lo;
            }
        }
        if (ent >= 0) {
            v = col_idx[ent];
            atomicCAS(hop_of + v, 0, hop + 2);
        }
    }
    slot_src[s] = u;
    slot_dst[s] = v;
    slot_ent[s] = ent;
}

__global__ void slot_flags(const int32_t* __restrict__ slot_dst, int64_t slots, int32_t* __restrict__ flags) {
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s > slots) return;
    flags[s] = (s < slots && slot_dst[s] >= 0) ? 1 : 0;
}

// Picks in slot order -> (local user, local item[, weight]); an entry that joins two nodes of the
// same side is reported through `bad`.
__global__ void emit_edges(const int32_t* __restrict__ slot_src, const int32_t* __restrict__ slot_dst,
                           const int32_t* __restrict__ slot_ent, const int32_t* __restrict__ pos, int64_t slots,
                           const int32_t* __restrict__ local_of, int32_t n_users, const float* __restrict__ val,
                           int32_t* __restrict__ edge_users, int32_t* __restrict__ edge_items,
                           float* __restrict__ edge_w, int32_t* __restrict__ bad) {
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= slots) return;
    const int32_t a = slot_src[s], b = slot_dst[s];
    if (b < 0) return;
    const int32_t user = a < b ? a : b, item = a < b ? b : a;
    const int32_t at = pos[s];
    if (user >= n_users || item < n_users) {
        atomicOr(bad, 2);
        edge_users[at] = 0;
        edge_items[at] = 0;
    } else {
        edge_users[at] = local_of[user];
        edge_items[at] = local_of[item] - local_of[n_users];
    }
    if (edge_w) edge_w[at] = val[slot_ent[s]];
}

__global__ void gather_counts(const int32_t* __restrict__ local_of, int32_t n_users, int32_t n,
                              const int32_t* __restrict__ n_edges, const int32_t* __restrict__ bad,
                              int32_t* __restrict__ out) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        out[0] = local_of[n_users];
        out[1] = local_of[n] - local_of[n_users];
        out[2] = *n_edges;
        out[3] = *bad;
    }
}

// Upper bounds that size the launches: cap_front[h] >= size of the frontier of hop h, slots[h] =
// cap_front[h] * fanout[h]; returns the total number of slots, or -1 when it does not fit int32.
int64_t plan(int64_t n, int64_t n_seeds, int32_t L, const int32_t* fanout, int64_t* cap_front, int64_t* slot_base) {
    int64_t total = 0, width = n_seeds < n ? n_seeds : n;
    for (int32_t h = 0; h < L; ++h) {
        cap_front[h] = width;
        slot_base[h] = total;
        const int64_t slots = width * fanout[h];
        total += slots;
        if (total > (int64_t)INT32_MAX - 1) return -1;
        width = slots < n ? slots : n;
    }
    return total;
}

int32_t check_plan(const char* who, int32_t n, int32_t n_seeds, int32_t L, const int32_t* h_fanout) {
    if (n < 0 || n_seeds < 0) return fail(E2EG_ERR_INVALID_ARG, "%s: negative size", who);
    if (L < 1 || L > kMaxHops) return fail(E2EG_ERR_INVALID_ARG, "%s: depth L=%d must be in [1, %d]", who, L, kMaxHops);
    if (!h_fanout) return fail(E2EG_ERR_NULL_PTR, "%s: h_fanout is null", who);
    for (int32_t h = 0; h < L; ++h)
        if (h_fanout[h] < 1 || h_fanout[h] > kMaxFanout)
            return fail(E2EG_ERR_INVALID_ARG, "%s: fan-out %d of hop %d must be in [1, %d]", who, h_fanout[h], h, kMaxFanout);
    return E2EG_OK;
}

struct SampleWs {
    int32_t* hop_of;    // [n + 1]
    int32_t* local_of;  // [n + 1] flags, then their prefix sums
    int32_t* frontier;  // [max cap_front]
    int32_t* slot_src;  // [slots]
    int32_t* slot_dst;
    int32_t* slot_ent;
    int32_t* slot_pos;  // [slots + 1]
    int32_t* small;     // [64]: [0..7] frontier sizes, [8] nodes, [9] edges, [10] bad, [16..19] counts for the host
    void* scan_ws;
    size_t bytes;
};

SampleWs carve_sample(void* base, int64_t n, int64_t max_front, int64_t slots) {
    Carver c(base);
    SampleWs w;
    w.hop_of = c.take<int32_t>(n + 1);
    w.local_of = c.take<int32_t>(n + 1);
    w.frontier = c.take<int32_t>(max_front > 0 ? max_front : 1);
    w.slot_src = c.take<int32_t>(slots > 0 ? slots : 1);
    w.slot_dst = c.take<int32_t>(slots > 0 ? slots : 1);
    w.slot_ent = c.take<int32_t>(slots > 0 ? slots : 1);
    w.slot_pos = c.take<int32_t>(slots + 1);
    w.small = c.take<int32_t>(64);
    const int64_t longest = (n + 1 > slots + 1) ? n + 1 : slots + 1;
    w.scan_ws = c.take<char>(scan_workspace_bytes(longest));
    w.bytes = c.size();
    return w;
}

}  // namespace
}  // namespace e2eg

using namespace e2eg;

extern "C" int32_t e2eg_sampling_weights(int64_t nnz, const float* d_val, float beta, float* d_p, void* stream_) {
    if (nnz < 0) return fail(E2EG_ERR_INVALID_ARG, "sampling_weights: negative size");
    if (!(beta >= 0.0f)) return fail(E2EG_ERR_INVALID_ARG, "sampling_weights: beta must be >= 0");
    if (nnz > 0 && (!d_val || !d_p)) return fail(E2EG_ERR_NULL_PTR, "sampling_weights: null pointer");
    if (nnz == 0) return E2EG_OK;
    pow_weights<<<grid_for(nnz), dim3(kThreads), 0, static_cast<hipStream_t>(stream_)>>>(d_val, nnz, beta, d_p);
    E2EG_LAUNCH_CHECK("pow_weights");
    return E2EG_OK;
}

extern "C" size_t e2eg_sampler_table_bytes(int64_t nnz) {
    if (nnz < 0) return 0;
    return align_up((size_t)(nnz + 1) * sizeof(uint64_t));
}

extern "C" size_t e2eg_sampler_prepare_workspace_bytes(int32_t n, int64_t nnz) {
    if (n < 0 || nnz < 0) return 0;
    return align_up((size_t)(n > 0 ? n : 1) * sizeof(int32_t)) + scan_u64_workspace_bytes(nnz + 1);   // row maxima, scan
}

extern "C" int32_t e2eg_sampler_prepare(int32_t n, int64_t nnz, const int32_t* d_row_ptr, const int32_t* d_col_idx,
                                        const float* d_p, void* d_table, size_t table_bytes, void* ws,
                                        size_t ws_bytes, void* stream_) {
    if (n < 0 || nnz < 0) return fail(E2EG_ERR_INVALID_ARG, "sampler_prepare: negative size");
    if (nnz > (int64_t)INT32_MAX || n == INT32_MAX)
        return fail(E2EG_ERR_OVERFLOW, "sampler_prepare: nnz=%lld exceeds int32", (long long)nnz);
    if (!d_row_ptr || !d_table || (nnz > 0 && (!d_col_idx || !d_p)))
        return fail(E2EG_ERR_NULL_PTR, "sampler_prepare: null pointer");
    if (nnz > 0 && n == 0) return fail(E2EG_ERR_INVALID_ARG, "sampler_prepare: entries given but no nodes");
    if (!aligned_to(d_table, kAlign) || table_bytes < e2eg_sampler_table_bytes(nnz))
        return fail(E2EG_ERR_CAPACITY, "sampler_prepare: d_table needs %zu bytes, 256-byte aligned",
                    e2eg_sampler_table_bytes(nnz));
    const size_t need = e2eg_sampler_prepare_workspace_bytes(n, nnz);
    if (!ws || !aligned_to(ws, kAlign) || ws_bytes < need)
        return fail(E2EG_ERR_WORKSPACE, "sampler_prepare: workspace needs %zu bytes, 256-byte aligned", need);
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    uint64_t* q = static_cast<uint64_t*>(d_table);
    int32_t* row_max_bits = static_cast<int32_t*>(ws);
    void* scan_ws = static_cast<char*>(ws) + align_up((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    const dim3 blk(kThreads);
    if (n > 0) {
        fill_i32<<<grid_for(n), blk, 0, stream>>>(row_max_bits, n, 0);
        E2EG_LAUNCH_CHECK("fill_i32");
    }
    if (nnz > 0) {
        row_max<<<grid_for(nnz), blk, 0, stream>>>(d_row_ptr, d_col_idx, d_p, n, nnz, row_max_bits);
        E2EG_LAUNCH_CHECK("row_max");
    }
    quantise_entries<<<grid_for(nnz + 1), blk, 0, stream>>>(d_row_ptr, d_col_idx, d_p, n, nnz, row_max_bits, q);
    E2EG_LAUNCH_CHECK("quantise_entries");
    E2EG_HIP_TRY(exclusive_scan_u64(q, q, nnz + 1, nullptr, scan_ws, stream));
    return E2EG_OK;
}

extern "C" int64_t e2eg_sample_capacity(int32_t n, int32_t n_seeds, int32_t L, const int32_t* h_fanout) {
    if (check_plan("sample_capacity", n, n_seeds, L, h_fanout) != E2EG_OK) return -1;
    int64_t cap_front[kMaxHops], slot_base[kMaxHops];
    const int64_t slots = plan(n, n_seeds, L, h_fanout, cap_front, slot_base);
    if (slots < 0) fail(E2EG_ERR_OVERFLOW, "sample_capacity: seeds x fan-outs exceed int32");
    return slots;
}

extern "C" size_t e2eg_sample_subgraph_workspace_bytes(int32_t n, int32_t n_seeds, int32_t L,
                                                       const int32_t* h_fanout) {
    if (check_plan("sample_subgraph_workspace_bytes", n, n_seeds, L, h_fanout) != E2EG_OK) return 0;
    int64_t cap_front[kMaxHops], slot_base[kMaxHops];
    const int64_t slots = plan(n, n_seeds, L, h_fanout, cap_front, slot_base);
    if (slots < 0) return 0;
    int64_t max_front = 0;
    for (int32_t h = 0; h < L; ++h) max_front = cap_front[h] > max_front ? cap_front[h] : max_front;
    return carve_sample(nullptr, n, max_front, slots).bytes;
}

extern "C" int32_t e2eg_sample_subgraph(int32_t n_users, int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                                        const int32_t* d_col_idx, const void* d_table, const float* d_val,
                                        int32_t n_seeds, const int32_t* d_seeds, int32_t L, const int32_t* h_fanout,
                                        uint64_t seed, int32_t* d_nodes, int64_t node_capacity,
                                        int32_t* d_edge_users, int32_t* d_edge_items, float* d_edge_w,
                                        int64_t edge_capacity, int32_t* h_counts, void* ws, size_t ws_bytes,
                                        void* stream_) {
    const char* who = "sample_subgraph";
    int32_t st = check_plan(who, n, n_seeds, L, h_fanout);
    if (st != E2EG_OK) return st;
    if (nnz < 0 || n_users < 0 || n_users > n) return fail(E2EG_ERR_INVALID_ARG, "%s: bad n_users or nnz", who);
    if (nnz > (int64_t)INT32_MAX || n == INT32_MAX)
        return fail(E2EG_ERR_OVERFLOW, "%s: nnz=%lld exceeds int32", who, (long long)nnz);
    if (!h_counts || !d_row_ptr || !d_table || (nnz > 0 && !d_col_idx) || (n_seeds > 0 && !d_seeds))
        return fail(E2EG_ERR_NULL_PTR, "%s: null pointer", who);
    if (d_edge_w && !d_val) return fail(E2EG_ERR_NULL_PTR, "%s: d_edge_w asks for weights but d_val is null", who);
    int64_t cap_front[kMaxHops], slot_base[kMaxHops];
    const int64_t slots = plan(n, n_seeds, L, h_fanout, cap_front, slot_base);
    if (slots < 0) return fail(E2EG_ERR_OVERFLOW, "%s: seeds x fan-outs exceed int32", who);
    const int64_t max_nodes = (int64_t)n_seeds + slots < n ? (int64_t)n_seeds + slots : n;
    if (node_capacity < max_nodes || edge_capacity < slots)
        return fail(E2EG_ERR_CAPACITY, "%s: needs room for %lld nodes and %lld edges", who, (long long)max_nodes,
                    (long long)slots);
    if ((max_nodes > 0 && !d_nodes) || (slots > 0 && (!d_edge_users || !d_edge_items)))
        return fail(E2EG_ERR_NULL_PTR, "%s: null output pointer", who);
    int64_t max_front = 0;
    for (int32_t h = 0; h < L; ++h) max_front = cap_front[h] > max_front ? cap_front[h] : max_front;
    const size_t need = carve_sample(nullptr, n, max_front, slots).bytes;
    if (!ws || !aligned_to(ws, kAlign) || ws_bytes < need)
        return fail(E2EG_ERR_WORKSPACE, "%s: workspace needs %zu bytes, 256-byte aligned", who, need);
    h_counts[0] = h_counts[1] = h_counts[2] = 0;
    if (n == 0 || n_seeds == 0) return E2EG_OK;

    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const SampleWs w = carve_sample(ws, n, max_front, slots);
    const uint64_t* cum = static_cast<const uint64_t*>(d_table);
    const dim3 blk(kThreads);
    fill_i32<<<grid_for((int64_t)n + 1), blk, 0, stream>>>(w.hop_of, (int64_t)n + 1, 0);
    E2EG_LAUNCH_CHECK("fill_i32");
    fill_i32<<<dim3(1), dim3(64), 0, stream>>>(w.small, 64, 0);
    E2EG_LAUNCH_CHECK("fill_i32");
    mark_seeds<<<grid_for(n_seeds), blk, 0, stream>>>(d_seeds, n_seeds, n, w.hop_of, w.small + 10);
    E2EG_LAUNCH_CHECK("mark_seeds");
    for (int32_t h = 0; h < L; ++h) {
        // the frontier of hop h, ascending: nodes whose mark is h + 1
        level_flags<<<grid_for((int64_t)n + 1), blk, 0, stream>>>(w.hop_of, n, h + 1, w.local_of);
        E2EG_LAUNCH_CHECK("level_flags");
        E2EG_HIP_TRY(exclusive_scan_i32(w.local_of, w.local_of, (int64_t)n + 1, w.small + h, w.scan_ws, stream));
        scatter_level<<<grid_for(n), blk, 0, stream>>>(w.hop_of, n, h + 1, w.local_of, w.frontier, cap_front[h]);
        E2EG_LAUNCH_CHECK("scatter_level");
        draw_picks<<<grid_for(cap_front[h] * h_fanout[h]), blk, 0, stream>>>(
            d_row_ptr, d_col_idx, cum, w.frontier, w.small + h, cap_front[h], h_fanout[h], h, (uint32_t)seed,
            (uint32_t)(seed >> 32), w.hop_of, w.slot_src + slot_base[h], w.slot_dst + slot_base[h],
            w.slot_ent + slot_base[h]);
        E2EG_LAUNCH_CHECK("draw_picks");
    }
    // local numbering: visited nodes in ascending order (users first, as in the parent)
    level_flags<<<grid_for((int64_t)n + 1), blk, 0, stream>>>(w.hop_of, n, 0, w.local_of);
    E2EG_LAUNCH_CHECK("level_flags");
    E2EG_HIP_TRY(exclusive_scan_i32(w.local_of, w.local_of, (int64_t)n + 1, w.small + 8, w.scan_ws, stream));
    scatter_level<<<grid_for(n), blk, 0, stream>>>(w.hop_of, n, 0, w.local_of, d_nodes, node_capacity);
    E2EG_LAUNCH_CHECK("scatter_level");
    // the picks, without the empty slots, in slot order
    slot_flags<<<grid_for(slots + 1), blk, 0, stream>>>(w.slot_dst, slots, w.slot_pos);
    E2EG_LAUNCH_CHECK("slot_flags");
    E2EG_HIP_TRY(exclusive_scan_i32(w.slot_pos, w.slot_pos, slots + 1, w.small + 9, w.scan_ws, stream));
    emit_edges<<<grid_for(slots), blk, 0, stream>>>(w.slot_src, w.slot_dst, w.slot_ent, w.slot_pos, slots, w.local_of,
                                                     n_users, d_val, d_edge_users, d_edge_items, d_edge_w, w.small + 10);
    E2EG_LAUNCH_CHECK("emit_edges");
    gather_counts<<<dim3(1), dim3(64), 0, stream>>>(w.local_of, n_users, n, w.small + 9, w.small + 10, w.small + 16);
    E2EG_LAUNCH_CHECK("gather_counts");
    int32_t host[4] = {0, 0, 0, 0};
    E2EG_HIP_TRY(hipMemcpyAsync(host, w.small + 16, sizeof(host), hipMemcpyDeviceToHost, stream));
    E2EG_HIP_TRY(hipStreamSynchronize(stream));  // the one wait: the counts size what the caller does next
    if (host[3] & 1) return fail(E2EG_ERR_BAD_INDEX, "%s: a seed is out of range", who);
    if (host[3] & 2) return fail(E2EG_ERR_BAD_INDEX, "%s: a stored entry joins two users or two items", who);
    h_counts[0] = host[0];
    h_counts[1] = host[1];
    h_counts[2] = host[2];
    return E2EG_OK;
}
