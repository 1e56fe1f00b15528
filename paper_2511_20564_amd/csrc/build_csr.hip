// e2eg_build_csr: (user, item) pairs -> CSR structure of A~ = A + I (paper: Section 3,
// "Notation"; A_ij > 0 iff (i,j) in E, so repeated pairs are one edge).
//
// Design for the GPU: everything is integer work and deterministic.
//   1. pack each pair into a 64-bit key (user << 32 | item), checking id ranges;
//   2. LSD radix sort (8-bit digits, only the bits the id ranges use) -> (user, item) order;
//   3. drop repeats (head flags, prefix sum, compaction) -> E distinct pairs;
//   4. user rows are read off directly: a user's items are a contiguous, ascending run;
//   5. swap the key halves and sort stably by item -> (item, user) order gives the item rows;
//   6. degrees come from run boundaries (no atomics), row_ptr from a prefix sum.
#include "common.h"

namespace e2eg {
namespace {

constexpr int kThreads = 256;

inline unsigned blocks_for(int64_t count, int per_block) {
    return (unsigned)ceil_div(count > 0 ? count : 1, per_block);
}

__global__ void fill_i32(int32_t* p, int64_t count, int32_t v) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = v;
}

__global__ void pack_pairs(const int32_t* __restrict__ users, const int32_t* __restrict__ items,
                           int64_t n_edges, int32_t n_users, int32_t n_items,
                           uint64_t* __restrict__ keys, int32_t* __restrict__ bad) {
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_edges) return;
    int32_t u = users[e], i = items[e];
    if (u < 0 || u >= n_users || i < 0 || i >= n_items) {
        atomicOr(bad, 1);
        u = 0;
        i = 0;
    }
    keys[e] = ((uint64_t)(uint32_t)u << 32) | (uint32_t)i;
}

__global__ void head_flags(const uint64_t* __restrict__ keys, int64_t count,
                           int32_t* __restrict__ flags) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < count) flags[k] = (k == 0 || keys[k] != keys[k - 1]) ? 1 : 0;
}

__global__ void compact_heads(const uint64_t* __restrict__ keys, int64_t count,
                              const int32_t* __restrict__ pos, uint64_t* __restrict__ out) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < count && (k == 0 || keys[k] != keys[k - 1])) out[pos[k]] = keys[k];
}

// Keys sorted by their upper half: record where each id's run starts and ends.
__global__ void run_bounds(const uint64_t* __restrict__ keys, int64_t count,
                           int32_t* __restrict__ start, int32_t* __restrict__ end) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= count) return;
    const uint32_t id = (uint32_t)(keys[k] >> 32);
    if (k == 0 || (uint32_t)(keys[k - 1] >> 32) != id) start[id] = (int32_t)k;
    if (k == count - 1 || (uint32_t)(keys[k + 1] >> 32) != id) end[id] = (int32_t)(k + 1);
}

// User rows: pair k of the (user, item)-sorted list lands behind its user's diagonal entry.
// Also rewrites the key as (item << 32 | user) for the second sort.
__global__ void fill_user_rows(uint64_t* __restrict__ keys, int64_t count, int32_t n_users,
                               int32_t self, int32_t* __restrict__ col_idx) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= count) return;
    const uint64_t key = keys[k];
    const uint32_t u = (uint32_t)(key >> 32), i = (uint32_t)key;
    col_idx[k + (int64_t)(u + 1) * self] = n_users + (int32_t)i;
    keys[k] = ((uint64_t)i << 32) | u;
}

__global__ void fill_item_rows(const uint64_t* __restrict__ keys, int64_t count, int32_t n_users,
                               int32_t self, int32_t* __restrict__ col_idx) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= count) return;
    const uint64_t key = keys[k];
    const uint32_t i = (uint32_t)(key >> 32), u = (uint32_t)key;
    col_idx[count + (int64_t)n_users * self + (int64_t)i * self + k] = (int32_t)u;
}

// counts[v] = run length (+1 with self-loops); counts[n] = 0 so the scan yields row_ptr[n].
// (in place: `end` becomes the counts)
__global__ void row_counts(const int32_t* __restrict__ start, int32_t* end, int64_t n,
                           int32_t self) {
    int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < n) end[v] = end[v] - start[v] + self;
    if (v == n) end[v] = 0;
}

__global__ void fill_diagonal(const int32_t* __restrict__ row_ptr, int64_t n, int32_t n_users,
                              int32_t* __restrict__ col_idx) {
    int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    // user row: itself first (items have larger ids); item row: itself last
    const int64_t at = v < n_users ? (int64_t)row_ptr[v] : (int64_t)row_ptr[v + 1] - 1;
    col_idx[at] = (int32_t)v;
}

// Weighted graphs (Section 3, "Notation": A_ij > 0 marks an edge, so its size is free to carry
// a strength).  Stored values of A~: 1 on the diagonal, 0 until a listed pair brings its weight.
__global__ void init_values(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                            int64_t n, int64_t nnz, float* __restrict__ val) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= nnz) return;
    int64_t lo = 0, hi = n - 1;  // the row of entry e: last i with row_ptr[i] <= e
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (row_ptr[mid] <= e) lo = mid; else hi = mid - 1;
    }
    val[e] = col_idx[e] == (int32_t)lo ? 1.0f : 0.0f;
}

// One thread per (pair, direction): the entry is found by binary search in its (ascending) row; a
// pair listed several times keeps its largest weight.  Positive floats order like their bit
// patterns read as integers, which makes the maximum an integer atomic and the result independent
// of the order of arrival.
__global__ void apply_weights(const int32_t* __restrict__ users, const int32_t* __restrict__ items,
                              const float* __restrict__ weights, int64_t n_edges, int32_t n_users,
                              int32_t n_items, const int32_t* __restrict__ row_ptr,
                              const int32_t* __restrict__ col_idx, float* val) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= 2 * n_edges) return;
    const int64_t e = t >> 1;
    const int32_t u = users[e], i = items[e];
    const float w = weights[e];
    if (u < 0 || u >= n_users || i < 0 || i >= n_items || !(w > 0.0f)) return;
    const int32_t r = (t & 1) ? n_users + i : u;
    const int32_t c = (t & 1) ? u : n_users + i;
    const int32_t end = row_ptr[r + 1];
    int32_t lo = row_ptr[r], hi = end;  // first position with col_idx >= c
    while (lo < hi) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        if (col_idx[mid] < c) lo = mid + 1; else hi = mid;
    }
    if (lo < end && col_idx[lo] == c) atomicMax(reinterpret_cast<int*>(val) + lo, __float_as_int(w));
}

struct BuildWs {
    uint64_t* buf_a;
    uint64_t* buf_b;
    int32_t* pos;
    void* sort_ws;
    int32_t* run_start;
    int32_t* run_end;
    int32_t* small;  // [0] distinct-pair count, [1] bad-id flag
    void* scan_ws;
    size_t bytes;
};

BuildWs carve_build(void* base, int32_t n_users, int32_t n_items, int64_t n_edges) {
    const int64_t n = (int64_t)n_users + n_items;
    const int64_t e = n_edges > 0 ? n_edges : 1;
    Carver c(base);
    BuildWs w;
    w.buf_a = c.take<uint64_t>(e);
    w.buf_b = c.take<uint64_t>(e);
    w.pos = c.take<int32_t>(e);
    w.sort_ws = c.take<char>(radix_sort_workspace_bytes(e));
    w.run_start = c.take<int32_t>(n + 1);
    w.run_end = c.take<int32_t>(n + 1);
    w.small = c.take<int32_t>(64);
    int64_t longest = e;
    if (n + 1 > longest) longest = n + 1;
    w.scan_ws = c.take<char>(scan_workspace_bytes(longest));
    w.bytes = c.size();
    return w;
}

}  // namespace
}  // namespace e2eg

using namespace e2eg;

extern "C" size_t e2eg_build_csr_workspace_bytes(int32_t n_users, int32_t n_items,
                                                 int64_t n_edges) {
    if (n_users < 0 || n_items < 0 || n_edges < 0) return 0;
    return carve_build(nullptr, n_users, n_items, n_edges).bytes;
}

extern "C" int32_t e2eg_build_csr(int32_t n_users, int32_t n_items, int64_t n_edges,
                                  const int32_t* d_user_ids, const int32_t* d_item_ids,
                                  int32_t flags, int32_t* d_row_ptr, int32_t* d_col_idx,
                                  int64_t col_capacity, int64_t* h_nnz_out, void* ws,
                                  size_t ws_bytes, void* stream_) {
    if (n_users < 0 || n_items < 0 || n_edges < 0)
        return fail(E2EG_ERR_INVALID_ARG, "build_csr: negative size");
    if (flags & ~E2EG_ADD_SELF_LOOPS) return fail(E2EG_ERR_INVALID_ARG, "build_csr: unknown flag bits 0x%x", flags);
    const int64_t n = (int64_t)n_users + n_items;
    const int32_t self = (flags & E2EG_ADD_SELF_LOOPS) ? 1 : 0;
    if (n > INT32_MAX - 1 || n_edges > (int64_t)INT32_MAX || 2 * n_edges + n > (int64_t)INT32_MAX)
        return fail(E2EG_ERR_OVERFLOW, "build_csr: n=%lld, 2*n_edges+n=%lld exceed int32",
                    (long long)n, (long long)(2 * n_edges + n));
    if (!d_row_ptr || !h_nnz_out || (n_edges > 0 && (!d_user_ids || !d_item_ids)))
        return fail(E2EG_ERR_NULL_PTR, "build_csr: null pointer");
    if ((2 * n_edges + n * self) > 0 && !d_col_idx)
        return fail(E2EG_ERR_NULL_PTR, "build_csr: d_col_idx is null");
    if (col_capacity < 2 * n_edges + n * self)
        return fail(E2EG_ERR_CAPACITY, "build_csr: col_capacity %lld < 2*n_edges+n = %lld",
                    (long long)col_capacity, (long long)(2 * n_edges + n * self));
    if (n_edges > 0 && (n_users == 0 || n_items == 0))
        return fail(E2EG_ERR_INVALID_ARG, "build_csr: edges given but no users or no items");
    const size_t need = e2eg_build_csr_workspace_bytes(n_users, n_items, n_edges);
    if (!ws || !aligned_to(ws, kAlign) || ws_bytes < need)
        return fail(E2EG_ERR_WORKSPACE, "build_csr: workspace needs %zu bytes, 256-byte aligned", need);

    hipStream_t stream = static_cast<hipStream_t>(stream_);
    BuildWs w = carve_build(ws, n_users, n_items, n_edges);
    const dim3 blk(kThreads);

    fill_i32<<<dim3(1), dim3(64), 0, stream>>>(w.small, 64, 0);
    E2EG_LAUNCH_CHECK("fill_i32");
    fill_i32<<<dim3(blocks_for(n + 1, kThreads)), blk, 0, stream>>>(w.run_start, n + 1, 0);
    fill_i32<<<dim3(blocks_for(n + 1, kThreads)), blk, 0, stream>>>(w.run_end, n + 1, 0);
    E2EG_LAUNCH_CHECK("fill_i32");

    uint64_t* src = w.buf_a;
    uint64_t* dst = w.buf_b;
    int32_t host_small[2] = {0, 0};
    if (n_edges > 0) {
        pack_pairs<<<dim3(blocks_for(n_edges, kThreads)), blk, 0, stream>>>(
            d_user_ids, d_item_ids, n_edges, n_users, n_items, src, w.small + 1);
        E2EG_LAUNCH_CHECK("pack_pairs");
        int32_t st = radix_sort_u64(&src, &dst, n_edges, 0, bits_for(n_items), w.sort_ws, stream);
        if (st != E2EG_OK) return st;
        st = radix_sort_u64(&src, &dst, n_edges, 32, bits_for(n_users), w.sort_ws, stream);
        if (st != E2EG_OK) return st;
        head_flags<<<dim3(blocks_for(n_edges, kThreads)), blk, 0, stream>>>(src, n_edges, w.pos);
        E2EG_LAUNCH_CHECK("head_flags");
        E2EG_HIP_TRY(exclusive_scan_i32(w.pos, w.pos, n_edges, w.small, w.scan_ws, stream));
        compact_heads<<<dim3(blocks_for(n_edges, kThreads)), blk, 0, stream>>>(src, n_edges, w.pos, dst);
        E2EG_LAUNCH_CHECK("compact_heads");
        uint64_t* t = src;
        src = dst;
        dst = t;
        E2EG_HIP_TRY(hipMemcpyAsync(host_small, w.small, sizeof(host_small), hipMemcpyDeviceToHost, stream));
    }
    E2EG_HIP_TRY(hipStreamSynchronize(stream));  // the one wait: the pair count sizes what follows
    if (host_small[1] != 0) return fail(E2EG_ERR_BAD_INDEX, "build_csr: a user or item id is out of range");
    const int64_t pairs = host_small[0];
    const int64_t nnz = 2 * pairs + n * self;
    *h_nnz_out = nnz;

    if (pairs > 0) {
        const dim3 grid(blocks_for(pairs, kThreads));
        run_bounds<<<grid, blk, 0, stream>>>(src, pairs, w.run_start, w.run_end);
        E2EG_LAUNCH_CHECK("run_bounds");
        fill_user_rows<<<grid, blk, 0, stream>>>(src, pairs, n_users, self, d_col_idx);
        E2EG_LAUNCH_CHECK("fill_user_rows");
        int32_t st = radix_sort_u64(&src, &dst, pairs, 32, bits_for(n_items), w.sort_ws, stream);
        if (st != E2EG_OK) return st;
        run_bounds<<<grid, blk, 0, stream>>>(src, pairs, w.run_start + n_users, w.run_end + n_users);
        E2EG_LAUNCH_CHECK("run_bounds");
        fill_item_rows<<<grid, blk, 0, stream>>>(src, pairs, n_users, self, d_col_idx);
        E2EG_LAUNCH_CHECK("fill_item_rows");
    }
    // row_ptr = exclusive scan of per-row counts
    row_counts<<<dim3(blocks_for(n + 1, kThreads)), blk, 0, stream>>>(w.run_start, w.run_end, n, self);
    E2EG_LAUNCH_CHECK("row_counts");
    E2EG_HIP_TRY(exclusive_scan_i32(w.run_end, d_row_ptr, n + 1, nullptr, w.scan_ws, stream));
    if (self && n > 0) {
        fill_diagonal<<<dim3(blocks_for(n, kThreads)), blk, 0, stream>>>(d_row_ptr, n, n_users, d_col_idx);
        E2EG_LAUNCH_CHECK("fill_diagonal");
    }
    return E2EG_OK;
}

extern "C" int32_t e2eg_edge_weights(int32_t n_users, int32_t n_items, int64_t n_edges,
                                     const int32_t* d_user_ids, const int32_t* d_item_ids,
                                     const float* d_weights, int64_t nnz, const int32_t* d_row_ptr,
                                     const int32_t* d_col_idx, float* d_val, void* stream_) {
    if (n_users < 0 || n_items < 0 || n_edges < 0 || nnz < 0)
        return fail(E2EG_ERR_INVALID_ARG, "edge_weights: negative size");
    const int64_t n = (int64_t)n_users + n_items;
    if (n > INT32_MAX - 1 || n_edges > (int64_t)INT32_MAX || nnz > (int64_t)INT32_MAX)
        return fail(E2EG_ERR_OVERFLOW, "edge_weights: n=%lld, nnz=%lld exceed int32", (long long)n, (long long)nnz);
    if (!d_row_ptr || (n_edges > 0 && (!d_user_ids || !d_item_ids || !d_weights)) || (nnz > 0 && (!d_col_idx || !d_val)))
        return fail(E2EG_ERR_NULL_PTR, "edge_weights: null pointer");
    if (nnz > 0 && n == 0) return fail(E2EG_ERR_INVALID_ARG, "edge_weights: entries given but no nodes");
    if (nnz == 0) return E2EG_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const dim3 blk(kThreads);
    init_values<<<dim3(blocks_for(nnz, kThreads)), blk, 0, stream>>>(d_row_ptr, d_col_idx, n, nnz, d_val);
    E2EG_LAUNCH_CHECK("init_values");
    if (n_edges > 0) {
        apply_weights<<<dim3(blocks_for(2 * n_edges, kThreads)), blk, 0, stream>>>(
            d_user_ids, d_item_ids, d_weights, n_edges, n_users, n_items, d_row_ptr, d_col_idx, d_val);
        E2EG_LAUNCH_CHECK("apply_weights");
    }
    return E2EG_OK;
}
