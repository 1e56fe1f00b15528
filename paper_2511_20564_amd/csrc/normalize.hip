// e2eg_normalize: d~_i = sum_j A~_ij and d~_i^-1/2 (paper: Section 3, "Notation"), and the
// private, renumbered copy of the graph that the propagation kernels read.
//
// Renumbering.  The kTopNodes nodes of highest degree get internal ids 0, 1, ... by descending
// degree (ties in node order); all other nodes follow in node order.  The CSR is rewritten in
// internal ids, rows in internal order, columns ascending.  What this buys on a power-law
// user-item graph:
//   - "is this neighbour popular" is one compare, and the feature rows of the most popular
//     nodes are one contiguous block (the propagation kernel stages it in LDS);
//   - every neighbour list starts with its popular entries;
//   - everything else keeps the caller's node order (users, then items), so at any time the
//     whole GPU gathers from the same side of the graph and the L2 caches hold one hot set.
// Rows of at most kShortMax entries are listed ordered by length inside blocks of kSortBlock
// consecutive rows (the kernel sums several of them side by side, so neighbours in the list should
// be equally long, while the block-wise order keeps the users-then-items progression).  Longer
// rows are cut into segments of kSegLen entries; the segments of rows with several are ordered by
// first column, so that segments which read the same stretch of feature rows can be run at the
// same time on the same L2 (the kernel deals the ordered list out to the XCDs in contiguous
// eighths); rows of one segment follow in row order.
// All of it is integer work: radix sorts and scans.  Nothing here depends on the feature width.
#include "common.h"

namespace e2eg {
namespace {

constexpr int kThreads = 256;

// Per node: degree, d^-1/2, and the sort key (larger degree first, then node id).
__global__ void row_stats(const int32_t* __restrict__ row_ptr, int64_t n, int32_t* __restrict__ deg,
                          float* __restrict__ dinv_sqrt, uint64_t* __restrict__ keys) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t d = row_ptr[i + 1] - row_ptr[i];
    if (deg) deg[i] = d;
    dinv_sqrt[i] = d > 0 ? (float)(1.0 / sqrt((double)d)) : 0.0f;
    keys[i] = ((uint64_t)(uint32_t)(0x7fffffff - d) << 32) | (uint32_t)i;
}

// Sorted (degree, node) keys -> is the node one of the kTopNodes most popular, and its rank.
__global__ void mark_top(const uint64_t* __restrict__ sorted, int64_t n, int32_t* __restrict__ rank_of,
                         int32_t* __restrict__ not_top) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p > n) return;
    if (p == n) {
        not_top[p] = 0;
        return;
    }
    const int32_t i = (int32_t)(uint32_t)sorted[p];
    rank_of[i] = (int32_t)p;
    not_top[i] = p < kTopNodes ? 0 : 1;
}

// others_before = exclusive scan of not_top over node ids.  Internal position: top nodes by
// rank, the others behind them in node order.  Also per internal row: its length, how it is cut,
// and the key that orders the short rows (block of kSortBlock rows, then length, then row).
__global__ void permute_nodes(const int32_t* __restrict__ rank_of, const int32_t* __restrict__ others_before,
                              const int32_t* __restrict__ row_ptr, int64_t n, int32_t* __restrict__ orig,
                              int32_t* __restrict__ zpos, int32_t* __restrict__ zdeg,
                              int32_t* __restrict__ nseg, int32_t* __restrict__ nslot,
                              int32_t* __restrict__ is_long, int32_t* __restrict__ is_multi,
                              uint64_t* __restrict__ short_keys) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n) return;
    if (i == n) {  // terminators so that the scans deliver the totals at index n
        zdeg[i] = 0;
        nseg[i] = 0;
        nslot[i] = 0;
        is_long[i] = 0;
        is_multi[i] = 0;
        return;
    }
    const int32_t n_top = n < kTopNodes ? (int32_t)n : kTopNodes;
    const int32_t r = rank_of[i];
    const int32_t p = r < kTopNodes ? r : n_top + others_before[i];
    const int32_t d = row_ptr[i + 1] - row_ptr[i];
    const int32_t segs = (d + kSegLen - 1) / kSegLen;
    orig[p] = (int32_t)i;
    zpos[i] = p;
    zdeg[p] = d;
    nseg[p] = d > kShortMax ? segs : 0;
    nslot[p] = d > kSegLen ? segs : 0;
    is_long[p] = d > kShortMax ? 1 : 0;
    is_multi[p] = d > kSegLen ? 1 : 0;
    const uint32_t hi = d > kShortMax ? 0x7fffffffu : (((uint32_t)p / kSortBlock) << 8) | (uint32_t)d;
    short_keys[p] = ((uint64_t)hi << 32) | (uint32_t)p;
}

struct RowScans {          // exclusive scans over internal rows, n + 1 entries each
    const int32_t* seg_off;
    const int32_t* slot_off;
    const int32_t* long_off;
    const int32_t* multi_off;
};

__global__ void emit_long_rows(const int32_t* __restrict__ zrow_ptr, RowScans sc, int64_t n, int64_t nnz,
                               SchedView s) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p > n) return;
    if (p == n) {
        SchedHeader h;
        h.n_long = sc.long_off[n];
        h.n_short = (int32_t)n - h.n_long;
        h.n_seg = sc.seg_off[n];
        h.n_multi = sc.multi_off[n];
        h.n_slot = sc.slot_off[n];
        h.n_seg_multi = h.n_slot;
        h.n = (int32_t)n;
        h.nnz = (int32_t)nnz;
        *s.header = h;
        s.seg_base[h.n_long] = h.n_seg;
        s.slot_base[h.n_multi] = h.n_slot;
        return;
    }
    const int32_t d = zrow_ptr[p + 1] - zrow_ptr[p];
    if (d > kShortMax) {
        const int32_t k = sc.long_off[p];  // < max_long: each such row has > kShortMax entries
        s.long_row[k] = (int32_t)p;
        s.seg_base[k] = sc.seg_off[p];
    }
    if (d > kSegLen) {
        const int32_t m = sc.multi_off[p];
        s.multi_row[m] = (int32_t)p;
        s.slot_base[m] = sc.slot_off[p];
    }
}

// One thread per segment t: find its row (binary search in the ascending segment bases),
// describe the segment, and key it for the ordering pass: slotted segments by first column, then
// the one-segment rows in row order.
__global__ void emit_segments(SchedView s, const int32_t* __restrict__ slot_off,
                              Segment* __restrict__ seg_tmp, uint64_t* __restrict__ keys) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int32_t n_seg = s.header->n_seg;
    if (t >= n_seg) return;
    int32_t lo = 0, hi = s.header->n_long - 1;  // last k with seg_base[k] <= t
    while (lo < hi) {
        const int32_t mid = (lo + hi + 1) >> 1;
        if (s.seg_base[mid] <= t) lo = mid; else hi = mid - 1;
    }
    const int32_t row = s.long_row[lo];
    const int32_t q = (int32_t)t - s.seg_base[lo];
    const int32_t row_beg = s.zrow_ptr[row], row_end = s.zrow_ptr[row + 1];
    const int32_t beg = row_beg + q * kSegLen;
    const int32_t end = beg + kSegLen < row_end ? beg + kSegLen : row_end;
    const bool multi = row_end - row_beg > kSegLen;
    seg_tmp[t] = Segment{row, beg, end, multi ? slot_off[row] + q : -1};
    keys[t] = multi ? ((uint64_t)(uint32_t)s.zcol[beg] << 32) | (uint32_t)t
                    : (1ull << 63) | ((uint64_t)(uint32_t)t << 32) | (uint32_t)t;
}

__global__ void fill_keys(uint64_t* __restrict__ keys, int64_t count) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < count) keys[k] = ~0ull;  // sorts behind every real segment
}

__global__ void place_segments(const uint64_t* __restrict__ keys, const Segment* __restrict__ seg_tmp,
                               SchedView s) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < s.header->n_seg) s.segs[p] = seg_tmp[(uint32_t)keys[p]];
}

__global__ void place_short_rows(const uint64_t* __restrict__ keys, int64_t n, SchedView s) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < n) s.short_rows[k] = (int32_t)(uint32_t)keys[k];  // the first n_short are the short rows
}

// One thread per CSR entry e: key = (internal row << bits) | internal column.
__global__ void entry_keys(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                           const int32_t* __restrict__ zpos, int64_t n, int64_t nnz, int bits,
                           uint64_t* __restrict__ keys) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= nnz) return;
    int64_t lo = 0, hi = n - 1;  // last i with row_ptr[i] <= e
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (row_ptr[mid] <= e) lo = mid; else hi = mid - 1;
    }
    keys[e] = ((uint64_t)(uint32_t)zpos[lo] << bits) | (uint32_t)zpos[col_idx[e]];
}

__global__ void unpack_columns(const uint64_t* __restrict__ keys, int64_t nnz, int bits,
                               int32_t* __restrict__ zcol) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < nnz) zcol[e] = (int32_t)(keys[e] & ((1ull << bits) - 1));
}

struct NormWs {
    uint64_t* keys_a;
    uint64_t* keys_b;
    int32_t* rank_of;
    int32_t* not_top;
    int32_t* zdeg;
    int32_t* nseg;
    int32_t* nslot;
    int32_t* is_long;
    int32_t* is_multi;
    Segment* seg_tmp;
    void* scan_ws;
    void* sort_ws;
    size_t bytes;
};

NormWs carve_norm(void* base, int64_t n, int64_t nnz) {
    Carver c(base);
    NormWs w;
    int64_t m = n + 1 > nnz ? n + 1 : nnz;
    if (sched_max_seg(nnz) > m) m = sched_max_seg(nnz);
    w.keys_a = c.take<uint64_t>(m);
    w.keys_b = c.take<uint64_t>(m);
    w.rank_of = c.take<int32_t>(n + 1);
    w.not_top = c.take<int32_t>(n + 1);
    w.zdeg = c.take<int32_t>(n + 1);
    w.nseg = c.take<int32_t>(n + 1);
    w.nslot = c.take<int32_t>(n + 1);
    w.is_long = c.take<int32_t>(n + 1);
    w.is_multi = c.take<int32_t>(n + 1);
    w.seg_tmp = c.take<Segment>(sched_max_seg(nnz));
    w.scan_ws = c.take<char>(scan_workspace_bytes(n + 1));
    w.sort_ws = c.take<char>(radix_sort_workspace_bytes(m));
    w.bytes = c.size();
    return w;
}

inline dim3 grid_for(int64_t count) { return dim3((unsigned)ceil_div(count > 0 ? count : 1, kThreads)); }

}  // namespace
}  // namespace e2eg

using namespace e2eg;

extern "C" size_t e2eg_sched_bytes(int32_t n, int64_t nnz) {
    if (n < 0 || nnz < 0) return 0;
    return sched_carve(nullptr, n, nnz, nullptr);
}

extern "C" size_t e2eg_normalize_workspace_bytes(int32_t n, int64_t nnz) {
    if (n < 0 || nnz < 0) return 0;
    return carve_norm(nullptr, n, nnz).bytes;
}

extern "C" int32_t e2eg_normalize(int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                                  const int32_t* d_col_idx, int32_t* d_deg, float* d_dinv_sqrt,
                                  void* d_sched, size_t sched_bytes, void* ws, size_t ws_bytes,
                                  void* stream_) {
    if (n < 0 || nnz < 0) return fail(E2EG_ERR_INVALID_ARG, "normalize: negative size");
    if (nnz > (int64_t)INT32_MAX || n == INT32_MAX)
        return fail(E2EG_ERR_OVERFLOW, "normalize: nnz=%lld exceeds int32", (long long)nnz);
    if (!d_row_ptr || !d_dinv_sqrt || !d_sched || (nnz > 0 && !d_col_idx))
        return fail(E2EG_ERR_NULL_PTR, "normalize: null pointer");
    if (!aligned_to(d_sched, kAlign) || sched_bytes < e2eg_sched_bytes(n, nnz))
        return fail(E2EG_ERR_CAPACITY, "normalize: d_sched needs %zu bytes, 256-byte aligned",
                    e2eg_sched_bytes(n, nnz));
    const size_t need = e2eg_normalize_workspace_bytes(n, nnz);
    if (!ws || !aligned_to(ws, kAlign) || ws_bytes < need)
        return fail(E2EG_ERR_WORKSPACE, "normalize: workspace needs %zu bytes, 256-byte aligned", need);

    hipStream_t stream = static_cast<hipStream_t>(stream_);
    NormWs w = carve_norm(ws, n, nnz);
    SchedView view;
    sched_carve(d_sched, n, nnz, &view);
    const dim3 blk(kThreads);

    // 1. degrees, d^-1/2, popularity order, internal numbering
    uint64_t* src = w.keys_a;
    uint64_t* dst = w.keys_b;
    if (n > 0) {
        row_stats<<<grid_for(n), blk, 0, stream>>>(d_row_ptr, n, d_deg, d_dinv_sqrt, src);
        E2EG_LAUNCH_CHECK("row_stats");
        int32_t st = radix_sort_u64(&src, &dst, n, 32, 32, w.sort_ws, stream);
        if (st != E2EG_OK) return st;
    }
    mark_top<<<grid_for((int64_t)n + 1), blk, 0, stream>>>(src, n, w.rank_of, w.not_top);
    E2EG_LAUNCH_CHECK("mark_top");
    E2EG_HIP_TRY(exclusive_scan_i32(w.not_top, w.not_top, (int64_t)n + 1, nullptr, w.scan_ws, stream));
    src = w.keys_a;
    dst = w.keys_b;
    permute_nodes<<<grid_for((int64_t)n + 1), blk, 0, stream>>>(w.rank_of, w.not_top, d_row_ptr, n, view.orig,
                                                               view.zpos, w.zdeg, w.nseg, w.nslot, w.is_long,
                                                               w.is_multi, src);
    E2EG_LAUNCH_CHECK("permute_nodes");
    if (n > 0) {  // short rows: by block of kSortBlock rows, then by length
        int32_t st = radix_sort_u64(&src, &dst, n, 32, 32, w.sort_ws, stream);
        if (st != E2EG_OK) return st;
        place_short_rows<<<grid_for(n), blk, 0, stream>>>(src, n, view);
        E2EG_LAUNCH_CHECK("place_short_rows");
    }
    E2EG_HIP_TRY(exclusive_scan_i32(w.zdeg, view.zrow_ptr, (int64_t)n + 1, nullptr, w.scan_ws, stream));
    E2EG_HIP_TRY(exclusive_scan_i32(w.nseg, w.nseg, (int64_t)n + 1, nullptr, w.scan_ws, stream));
    E2EG_HIP_TRY(exclusive_scan_i32(w.nslot, w.nslot, (int64_t)n + 1, nullptr, w.scan_ws, stream));
    E2EG_HIP_TRY(exclusive_scan_i32(w.is_long, w.is_long, (int64_t)n + 1, nullptr, w.scan_ws, stream));
    E2EG_HIP_TRY(exclusive_scan_i32(w.is_multi, w.is_multi, (int64_t)n + 1, nullptr, w.scan_ws, stream));

    // 2. the CSR in internal ids
    if (nnz > 0) {
        const int bits = bits_for(n);
        src = w.keys_a;
        dst = w.keys_b;
        entry_keys<<<grid_for(nnz), blk, 0, stream>>>(d_row_ptr, d_col_idx, view.zpos, n, nnz, bits, src);
        E2EG_LAUNCH_CHECK("entry_keys");
        int32_t st = radix_sort_u64(&src, &dst, nnz, 0, 2 * bits, w.sort_ws, stream);
        if (st != E2EG_OK) return st;
        unpack_columns<<<grid_for(nnz), blk, 0, stream>>>(src, nnz, bits, view.zcol);
        E2EG_LAUNCH_CHECK("unpack_columns");
    }

    // 3. long rows and their segments
    const RowScans sc{w.nseg, w.nslot, w.is_long, w.is_multi};
    emit_long_rows<<<grid_for((int64_t)n + 1), blk, 0, stream>>>(view.zrow_ptr, sc, n, nnz, view);
    E2EG_LAUNCH_CHECK("emit_long_rows");
    if (nnz > kShortMax) {  // otherwise no row can be long
        src = w.keys_a;
        dst = w.keys_b;
        fill_keys<<<grid_for(view.max_seg), blk, 0, stream>>>(src, view.max_seg);
        E2EG_LAUNCH_CHECK("fill_keys");
        emit_segments<<<grid_for(view.max_seg), blk, 0, stream>>>(view, w.nslot, w.seg_tmp, src);
        E2EG_LAUNCH_CHECK("emit_segments");
        int32_t st = radix_sort_u64(&src, &dst, view.max_seg, 32, 32, w.sort_ws, stream);
        if (st != E2EG_OK) return st;
        place_segments<<<grid_for(view.max_seg), blk, 0, stream>>>(src, w.seg_tmp, view);
        E2EG_LAUNCH_CHECK("place_segments");
    }
    return E2EG_OK;
}
