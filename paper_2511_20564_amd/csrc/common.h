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

// ---- device-wide exclusive scan (scan.hip) -------------------------------------------------
// out[i] = sum(in[0..i-1]); in == out allowed.  If d_total != nullptr the grand total is stored
// there.  `ws` needs scan_workspace_bytes(count).  Enqueued on `stream`.
size_t scan_workspace_bytes(int64_t count);
hipError_t exclusive_scan_i32(const int32_t* in, int32_t* out, int64_t count, int32_t* d_total,
                              void* ws, hipStream_t stream);

// ---- schedule layout shared by normalize.hip (writer) and propagate.hip (reader) ----------
constexpr int kSegLen = 512;  // longest run of CSR entries one wavefront sums

struct SchedHeader {
    int32_t n_items;    // work items (row segments)
    int32_t n_split;    // rows cut into more than one segment
    int32_t n_slots;    // partial-sum slots (= segments of split rows)
    int32_t seg_len;
    int32_t n;          // rows the schedule was built for
    int32_t nnz;
    int32_t pad[2];
};

struct SchedView {
    SchedHeader* header;
    int32_t* item_row;    // [max_items]
    int32_t* item_beg;    // [max_items] first CSR entry of the segment
    int32_t* item_slot;   // [max_items] partial slot, -1 when the segment is the whole row
    int32_t* split_row;   // [max_split]
    int32_t* split_base;  // [max_split] first slot
    int32_t* split_cnt;   // [max_split] number of slots
    int64_t max_items, max_split;
};

inline int64_t sched_max_items(int64_t n, int64_t nnz) { return n + nnz / kSegLen + 1; }
inline int64_t sched_max_split(int64_t nnz) { return nnz / kSegLen + 1; }
size_t sched_carve(void* base, int64_t n, int64_t nnz, SchedView* view);

}  // namespace e2eg
