// Shared host-side plumbing of libe2eg: error reporting, workspace carving, launch helpers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stddef.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/e2eg.h"

namespace e2eg {

// Thread-local message for e2eg_last_error().
void set_error(const char* fmt, ...);
int32_t fail(int32_t status, const char* fmt, ...);

#define E2EG_HIP_TRY(expr)                                                                   \
    do {                                                                                     \
        hipError_t e2eg_err_ = (expr);                                                       \
        if (e2eg_err_ != hipSuccess)                                                         \
            return ::e2eg::fail(E2EG_ERR_HIP, "%s failed: %s (%s:%d)", #expr,               \
                                hipGetErrorString(e2eg_err_), __FILE__, __LINE__);           \
    } while (0)

#define E2EG_LAUNCH_CHECK(name)                                                              \
    do {                                                                                     \
        hipError_t e2eg_err_ = hipGetLastError();                                            \
        if (e2eg_err_ != hipSuccess)                                                         \
            return ::e2eg::fail(E2EG_ERR_HIP, "launch of %s failed: %s", name,              \
                                hipGetErrorString(e2eg_err_));                               \
    } while (0)

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Carves aligned pieces out of a caller-provided workspace; `size()` with a null base is the
// sizing pass used by the *_workspace_bytes queries.
class Carver {
  public:
    explicit Carver(void* base) : base_(static_cast<char*>(base)), off_(0) {}
    template <typename T>
    T* take(size_t count) {
        size_t at = off_;
        off_ += align_up(count * sizeof(T));
        return base_ ? reinterpret_cast<T*>(base_ + at) : nullptr;
    }
    size_t size() const { return off_; }

  private:
    char* base_;
    size_t off_;
};

inline bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// ---- kernel timing for the measurement aid (status.hip) ------------------------------------
// profile_mark(stream, false) before and profile_mark(stream, true) after a launch; no-ops
// unless e2eg_profile_begin() is active on this thread.
void profile_mark(hipStream_t stream, bool after);

// ---- device-wide exclusive scan (scan.hip) -------------------------------------------------
// out[i] = sum(in[0..i-1]); in == out allowed.  If d_total != nullptr the grand total is stored
// there.  `ws` needs scan_workspace_bytes(count).  Enqueued on `stream`.
size_t scan_workspace_bytes(int64_t count);
hipError_t exclusive_scan_i32(const int32_t* in, int32_t* out, int64_t count, int32_t* d_total,
                              void* ws, hipStream_t stream);

// ---- stable LSD radix sort of 64-bit keys (sort.hip) ---------------------------------------
// Sorts by bits [lo, lo + nbits) only, 8 bits per pass, ping-ponging between *src and *dst; on
// return *src points at the sorted keys.  `ws` needs radix_sort_workspace_bytes(count).
size_t radix_sort_workspace_bytes(int64_t count);
int32_t radix_sort_u64(uint64_t** src, uint64_t** dst, int64_t count, int lo, int nbits, void* ws,
                       hipStream_t stream);
int bits_for(int64_t count);  // bits needed to represent ids 0 .. count-1 (at least 1)

// ---- schedule layout shared by normalize.hip (writer) and propagate.hip (reader) ----------
constexpr int kSegLen = 512;       // longest run of CSR entries one wavefront sums
constexpr int kShortPerWave = 4;   // whole (unsplit) rows a wavefront handles in one go
constexpr int kWavesPerBlock = 4;  // 256-thread workgroups

struct alignas(16) WorkItem {
    int32_t row;   // < 0: padding, nothing to do
    int32_t beg;   // first CSR entry
    int32_t end;   // one past the last CSR entry
    int32_t slot;  // partial-sum slot, or -1 when the item is a whole row
};

struct SchedHeader {
    int32_t n_short;  // rows with at most kSegLen entries (one work item each)
    int32_t n_seg;    // segments of the longer rows (= partial-sum slots)
    int32_t n_split;  // rows cut into segments
    int32_t seg_len;
    int32_t n;
    int32_t nnz;
    int32_t pad[2];
};

struct SchedView {
    SchedHeader* header;
    WorkItem* seg_items;    // [max_seg_pos] segments of long rows, placed for L2 locality; padded
    WorkItem* short_items;  // [n] whole rows in node order
    int32_t* split_row;     // [max_split]
    int32_t* split_base;    // [max_split] first slot
    int32_t* split_cnt;     // [max_split] number of slots
    int64_t max_seg, max_seg_pos, max_split;
};

// Upper bounds that depend on (n, nnz) only, so that launches need no device read-back.
inline int64_t sched_max_split(int64_t nnz) { return nnz / kSegLen + 1; }
inline int64_t sched_max_seg(int64_t nnz) { return 2 * (nnz / kSegLen) + 2; }
// Positions in seg_items: room for the per-XCD rounding of the placement, and a whole number of
// workgroups, so that every wavefront of the segment part of the grid reads an initialised record.
inline int64_t sched_max_seg_pos(int64_t nnz) {
    return (sched_max_seg(nnz) + 64 + kWavesPerBlock - 1) / kWavesPerBlock * kWavesPerBlock;
}
size_t sched_carve(void* base, int64_t n, int64_t nnz, SchedView* view);

}  // namespace e2eg
