// e2eg_normalize: d~_i = sum_j A~_ij and d~_i^-1/2 (paper: Section 3, "Notation"), and the row
// schedule for the propagation kernels.
//
// Schedule.  Rows with at most kSegLen entries ("short") are one work item each, kept in node
// order.  Longer rows (the power-law head: popular items whose neighbour lists sweep most of the
// user range) are cut into segments of kSegLen entries; each segment is summed by one wavefront
// into a numbered partial-sum slot and the slots of a row are added in slot order afterwards, so
// results do not depend on timing.  Segments are ordered by their first column and the ordered
// list is dealt out so that every XCD (workgroup index mod 8) gets one contiguous eighth of it:
// segments that read the same stretch of feature rows then run at the same time on the same
// L2, instead of each popular item streaming the whole feature table through every L2.
#include "common.h"

namespace e2eg {
namespace {

constexpr int kThreads = 256;
constexpr int kXcds = 8;

__global__ void row_stats(const int32_t* __restrict__ row_ptr, int64_t n,
                          int32_t* __restrict__ deg, float* __restrict__ dinv_sqrt,
                          int32_t* __restrict__ is_short, int32_t* __restrict__ slot_cnt,
                          int32_t* __restrict__ is_split) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n) return;
    if (i == n) {  // terminators so that the scans deliver the totals at index n
        is_short[i] = 0;
        slot_cnt[i] = 0;
        is_split[i] = 0;
        return;
    }
    const int32_t d = row_ptr[i + 1] - row_ptr[i];
    if (deg) deg[i] = d;
    dinv_sqrt[i] = d > 0 ? (float)(1.0 / sqrt((double)d)) : 0.0f;
    const bool split = d > kSegLen;
    is_short[i] = split ? 0 : 1;
    slot_cnt[i] = split ? (d + kSegLen - 1) / kSegLen : 0;
    is_split[i] = split ? 1 : 0;
}

__global__ void fill_padding(WorkItem* __restrict__ items, int64_t count) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < count) items[k] = WorkItem{-1, 0, 0, -1};
}

__global__ void fill_keys(uint64_t* __restrict__ keys, int64_t count) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < count) keys[k] = ~0ull;  // sorts behind every real segment
}

// One thread per row: short rows become work items; long rows are listed with their slot range.
__global__ void emit_rows(const int32_t* __restrict__ row_ptr, int64_t n, int64_t nnz,
                          const int32_t* __restrict__ short_off,
                          const int32_t* __restrict__ slot_off,
                          const int32_t* __restrict__ split_idx, SchedView s) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n) return;
    if (i == n) {
        SchedHeader h;
        h.n_short = short_off[n];
        h.n_seg = slot_off[n];
        h.n_split = split_idx[n];
        h.seg_len = kSegLen;
        h.n = (int32_t)n;
        h.nnz = (int32_t)nnz;
        h.pad[0] = h.pad[1] = 0;
        *s.header = h;
        return;
    }
    const int32_t beg = row_ptr[i], end = row_ptr[i + 1];
    const int32_t d = end - beg;
    if (d <= kSegLen) {
        s.short_items[short_off[i]] = WorkItem{(int32_t)i, beg, end, -1};
    } else {
        const int32_t k = split_idx[i];
        s.split_row[k] = (int32_t)i;
        s.split_base[k] = slot_off[i];
        s.split_cnt[k] = (d + kSegLen - 1) / kSegLen;
    }
}

// One thread per segment slot t: find its row (binary search in the ascending slot bases),
// describe the segment, and key it by its first column for the ordering pass.
__global__ void emit_segments(const int32_t* __restrict__ row_ptr,
                              const int32_t* __restrict__ col_idx, SchedView s,
                              WorkItem* __restrict__ seg_tmp, uint64_t* __restrict__ keys) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int32_t n_seg = s.header->n_seg;
    if (t >= n_seg) return;
    int32_t lo = 0, hi = s.header->n_split - 1;  // last k with split_base[k] <= t
    while (lo < hi) {
        const int32_t mid = (lo + hi + 1) >> 1;
        if (s.split_base[mid] <= t) lo = mid; else hi = mid - 1;
    }
    const int32_t row = s.split_row[lo];
    const int32_t q = (int32_t)t - s.split_base[lo];
    const int32_t beg = row_ptr[row] + q * kSegLen;
    const int32_t row_end = row_ptr[row + 1];
    const int32_t end = beg + kSegLen < row_end ? beg + kSegLen : row_end;
    seg_tmp[t] = WorkItem{row, beg, end, (int32_t)t};
    keys[t] = ((uint64_t)(uint32_t)col_idx[beg] << 32) | (uint32_t)t;
}

// Ordered position p -> place in seg_items such that XCD x (workgroup index mod 8) owns the
// x-th contiguous eighth of the ordered list.
__global__ void place_segments(const uint64_t* __restrict__ keys,
                               const WorkItem* __restrict__ seg_tmp, SchedView s) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int32_t n_seg = s.header->n_seg;
    if (p >= n_seg) return;
    int64_t per = (n_seg + kXcds - 1) / kXcds;
    per = (per + kWavesPerBlock - 1) / kWavesPerBlock * kWavesPerBlock;
    const int64_t xcd = p / per, r = p % per;
    const int64_t pos = ((r / kWavesPerBlock) * kXcds + xcd) * kWavesPerBlock + r % kWavesPerBlock;
    s.seg_items[pos] = seg_tmp[(uint32_t)keys[p]];
}

struct NormWs {
    int32_t* is_short;
    int32_t* slot_cnt;
    int32_t* is_split;
    WorkItem* seg_tmp;
    uint64_t* keys_a;
    uint64_t* keys_b;
    void* scan_ws;
    void* sort_ws;
    size_t bytes;
};

NormWs carve_norm(void* base, int64_t n, int64_t nnz) {
    Carver c(base);
    NormWs w;
    const int64_t max_seg = sched_max_seg(nnz);
    w.is_short = c.take<int32_t>(n + 1);
    w.slot_cnt = c.take<int32_t>(n + 1);
    w.is_split = c.take<int32_t>(n + 1);
    w.seg_tmp = c.take<WorkItem>(max_seg);
    w.keys_a = c.take<uint64_t>(max_seg);
    w.keys_b = c.take<uint64_t>(max_seg);
    w.scan_ws = c.take<char>(scan_workspace_bytes(n + 1));
    w.sort_ws = c.take<char>(radix_sort_workspace_bytes(max_seg));
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
    row_stats<<<grid_for((int64_t)n + 1), blk, 0, stream>>>(d_row_ptr, n, d_deg, d_dinv_sqrt, w.is_short,
                                                           w.slot_cnt, w.is_split);
    E2EG_LAUNCH_CHECK("row_stats");
    E2EG_HIP_TRY(exclusive_scan_i32(w.is_short, w.is_short, (int64_t)n + 1, nullptr, w.scan_ws, stream));
    E2EG_HIP_TRY(exclusive_scan_i32(w.slot_cnt, w.slot_cnt, (int64_t)n + 1, nullptr, w.scan_ws, stream));
    E2EG_HIP_TRY(exclusive_scan_i32(w.is_split, w.is_split, (int64_t)n + 1, nullptr, w.scan_ws, stream));
    fill_padding<<<grid_for(view.max_seg_pos), blk, 0, stream>>>(view.seg_items, view.max_seg_pos);
    E2EG_LAUNCH_CHECK("fill_padding");
    fill_keys<<<grid_for(view.max_seg), blk, 0, stream>>>(w.keys_a, view.max_seg);
    E2EG_LAUNCH_CHECK("fill_keys");
    emit_rows<<<grid_for((int64_t)n + 1), blk, 0, stream>>>(d_row_ptr, n, nnz, w.is_short, w.slot_cnt,
                                                           w.is_split, view);
    E2EG_LAUNCH_CHECK("emit_rows");
    if (nnz > kSegLen) {  // otherwise no row can be long
        emit_segments<<<grid_for(view.max_seg), blk, 0, stream>>>(d_row_ptr, d_col_idx, view, w.seg_tmp,
                                                                  w.keys_a);
        E2EG_LAUNCH_CHECK("emit_segments");
        uint64_t* src = w.keys_a;
        uint64_t* dst = w.keys_b;
        int32_t st = radix_sort_u64(&src, &dst, view.max_seg, 32, bits_for(n), w.sort_ws, stream);
        if (st != E2EG_OK) return st;
        place_segments<<<grid_for(view.max_seg), blk, 0, stream>>>(src, w.seg_tmp, view);
        E2EG_LAUNCH_CHECK("place_segments");
    }
    return E2EG_OK;
}
