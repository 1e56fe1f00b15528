// e2eg_normalize: d~_i = sum_j A~_ij and d~_i^-1/2 (paper: Section 3, "Notation"), and the row
// schedule for the propagation kernels.
//
// The schedule cuts every row into segments of at most kSegLen CSR entries.  A row that fits
// in one segment is summed and written by one wavefront; a longer (power-law head) row is
// spread over many wavefronts that leave fp32 partial sums in numbered slots, added up in a
// fixed order afterwards, so results do not depend on timing.
#include "common.h"

namespace e2eg {
namespace {

constexpr int kThreads = 256;

__global__ void row_stats(const int32_t* __restrict__ row_ptr, int64_t n,
                          int32_t* __restrict__ deg, float* __restrict__ dinv_sqrt,
                          int32_t* __restrict__ seg_cnt, int32_t* __restrict__ slot_cnt,
                          int32_t* __restrict__ is_split) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n) return;
    if (i == n) {  // terminators so that the scans deliver the totals at index n
        seg_cnt[i] = 0;
        slot_cnt[i] = 0;
        is_split[i] = 0;
        return;
    }
    const int32_t d = row_ptr[i + 1] - row_ptr[i];
    if (deg) deg[i] = d;
    dinv_sqrt[i] = d > 0 ? (float)(1.0 / sqrt((double)d)) : 0.0f;
    const int32_t segs = d <= kSegLen ? 1 : (d + kSegLen - 1) / kSegLen;
    seg_cnt[i] = segs;
    slot_cnt[i] = segs > 1 ? segs : 0;
    is_split[i] = segs > 1 ? 1 : 0;
}

__global__ void emit_schedule(const int32_t* __restrict__ row_ptr, int64_t n, int64_t nnz,
                              const int32_t* __restrict__ item_off,
                              const int32_t* __restrict__ slot_off,
                              const int32_t* __restrict__ split_idx, SchedView s) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n) return;
    if (i == n) {
        SchedHeader h;
        h.n_items = item_off[n];
        h.n_slots = slot_off[n];
        h.n_split = split_idx[n];
        h.seg_len = kSegLen;
        h.n = (int32_t)n;
        h.nnz = (int32_t)nnz;
        h.pad[0] = h.pad[1] = 0;
        *s.header = h;
        return;
    }
    const int32_t beg = row_ptr[i];
    const int32_t d = row_ptr[i + 1] - beg;
    const int32_t io = item_off[i];
    if (d <= kSegLen) {
        s.item_row[io] = (int32_t)i;
        s.item_beg[io] = beg;
        s.item_slot[io] = -1;
        return;
    }
    const int32_t segs = (d + kSegLen - 1) / kSegLen;
    const int32_t so = slot_off[i];
    const int32_t si = split_idx[i];
    s.split_row[si] = (int32_t)i;
    s.split_base[si] = so;
    s.split_cnt[si] = segs;
    for (int32_t k = 0; k < segs; ++k) {
        s.item_row[io + k] = (int32_t)i;
        s.item_beg[io + k] = beg + k * kSegLen;
        s.item_slot[io + k] = so + k;
    }
}

struct NormWs {
    int32_t* seg_cnt;
    int32_t* slot_cnt;
    int32_t* is_split;
    void* scan_ws;
    size_t bytes;
};

NormWs carve_norm(void* base, int64_t n) {
    Carver c(base);
    NormWs w;
    w.seg_cnt = c.take<int32_t>(n + 1);
    w.slot_cnt = c.take<int32_t>(n + 1);
    w.is_split = c.take<int32_t>(n + 1);
    w.scan_ws = c.take<char>(scan_workspace_bytes(n + 1));
    w.bytes = c.size();
    return w;
}

}  // namespace
}  // namespace e2eg

using namespace e2eg;

extern "C" size_t e2eg_sched_bytes(int32_t n, int64_t nnz) {
    if (n < 0 || nnz < 0) return 0;
    return sched_carve(nullptr, n, nnz, nullptr);
}

extern "C" size_t e2eg_normalize_workspace_bytes(int32_t n, int64_t nnz) {
    (void)nnz;
    if (n < 0) return 0;
    return carve_norm(nullptr, n).bytes;
}

extern "C" int32_t e2eg_normalize(int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                                  int32_t* d_deg, float* d_dinv_sqrt, void* d_sched,
                                  size_t sched_bytes, void* ws, size_t ws_bytes, void* stream_) {
    if (n < 0 || nnz < 0) return fail(E2EG_ERR_INVALID_ARG, "normalize: negative size");
    if (nnz > (int64_t)INT32_MAX || n == INT32_MAX)
        return fail(E2EG_ERR_OVERFLOW, "normalize: nnz=%lld exceeds int32", (long long)nnz);
    if (!d_row_ptr || !d_dinv_sqrt || !d_sched) return fail(E2EG_ERR_NULL_PTR, "normalize: null pointer");
    if (!aligned_to(d_sched, kAlign) || sched_bytes < e2eg_sched_bytes(n, nnz))
        return fail(E2EG_ERR_CAPACITY, "normalize: d_sched needs %zu bytes, 256-byte aligned",
                    e2eg_sched_bytes(n, nnz));
    const size_t need = e2eg_normalize_workspace_bytes(n, nnz);
    if (!ws || !aligned_to(ws, kAlign) || ws_bytes < need)
        return fail(E2EG_ERR_WORKSPACE, "normalize: workspace needs %zu bytes, 256-byte aligned", need);

    hipStream_t stream = static_cast<hipStream_t>(stream_);
    NormWs w = carve_norm(ws, n);
    SchedView view;
    sched_carve(d_sched, n, nnz, &view);
    const dim3 blk(kThreads);
    const dim3 grid((unsigned)ceil_div((int64_t)n + 1, kThreads));
    row_stats<<<grid, blk, 0, stream>>>(d_row_ptr, n, d_deg, d_dinv_sqrt, w.seg_cnt, w.slot_cnt, w.is_split);
    E2EG_LAUNCH_CHECK("row_stats");
    E2EG_HIP_TRY(exclusive_scan_i32(w.seg_cnt, w.seg_cnt, (int64_t)n + 1, nullptr, w.scan_ws, stream));
    E2EG_HIP_TRY(exclusive_scan_i32(w.slot_cnt, w.slot_cnt, (int64_t)n + 1, nullptr, w.scan_ws, stream));
    E2EG_HIP_TRY(exclusive_scan_i32(w.is_split, w.is_split, (int64_t)n + 1, nullptr, w.scan_ws, stream));
    emit_schedule<<<grid, blk, 0, stream>>>(d_row_ptr, n, nnz, w.seg_cnt, w.slot_cnt, w.is_split, view);
    E2EG_LAUNCH_CHECK("emit_schedule");
    return E2EG_OK;
}
