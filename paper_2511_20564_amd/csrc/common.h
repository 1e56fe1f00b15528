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

// ---- schedule shared by normalize.hip (writer) and propagate.hip (reader) ------------------
// The propagation kernels work on a private copy of the graph with renumbered nodes ("internal"
// ids): the kTopNodes nodes of highest degree come first, by descending degree (ties in node
// order); all other nodes follow in node order.  Popular nodes, whose feature rows are read most
// often, so have the lowest ids, sit at the front of every neighbour list, and their feature rows
// are one contiguous block.
//
// Work is cut in two ways.  Rows with at most kShortMax entries ("short") are listed in
// `short_rows`, ordered by length inside blocks of kSortBlock consecutive rows: a wavefront
// sums several short rows side by side (one lane group per row), and neighbours in that list
// have similar lengths.  Longer rows are cut into segments of kSegLen entries, one wavefront
// each; a row of one segment is finished by that wavefront, a row of several leaves numbered fp32
// partial sums ("slots") that are added in slot order afterwards.
constexpr int kShortMax = 128;         // longest row summed by a single lane group
constexpr int kSegLen = 512;           // longest run of CSR entries summed by one wavefront
constexpr int kSortBlock = 4096;       // short rows are ordered by length within such blocks
constexpr int kHotBytes = 128 * 1024;  // feature rows of the most popular nodes kept in LDS
constexpr int kTopNodes = kHotBytes / 16;  // most rows that can be staged (16-byte rows)

struct alignas(16) Segment {
    int32_t row;   // internal row
    int32_t beg;   // first entry in zcol
    int32_t end;   // one past the last entry
    int32_t slot;  // partial-sum slot, or -1 when the segment is the whole row
};

struct SchedHeader {
    int32_t n_short;  // rows with at most kShortMax entries
    int32_t n_long;   // rows with more
    int32_t n_seg;    // segments of those rows
    int32_t n_multi;  // rows with more than kSegLen entries (several segments)
    int32_t n_slot;   // segments of those rows (= partial-sum slots)
    int32_t n_seg_multi;  // = n_slot: the first n_slot entries of `segs` are the slotted ones
    int32_t n;
    int32_t nnz;
};

struct SchedView {
    SchedHeader* header;
    int32_t* orig;        // [n] node at internal position p
    int32_t* zpos;        // [n] internal position of node i
    int32_t* zrow_ptr;    // [n + 1] row pointers of the internal CSR
    int32_t* zcol;        // [nnz] internal column ids, ascending within each row
    int32_t* short_rows;  // [n] internal rows with at most kShortMax entries, processing order
    int32_t* long_row;    // [max_long] internal rows with more than kShortMax entries, ascending
    int32_t* seg_base;    // [max_long + 1] first segment number of each long row
    int32_t* multi_row;   // [max_multi] internal rows with more than kSegLen entries, ascending
    int32_t* slot_base;   // [max_multi + 1] first slot of each such row; [n_multi] = n_slot
    Segment* segs;        // [max_seg]: slotted segments ordered by first column, then one-segment rows
    int64_t max_long, max_seg, max_multi, max_slot;
};

// Upper bounds that depend on nnz only, so that launches need no device read-back.
inline int64_t sched_max_long(int64_t nnz) { return nnz / (kShortMax + 1) + 1; }
inline int64_t sched_max_seg(int64_t nnz) { return nnz / kSegLen + sched_max_long(nnz) + 1; }
inline int64_t sched_max_multi(int64_t nnz) { return nnz / (kSegLen + 1) + 1; }
inline int64_t sched_max_slot(int64_t nnz) { return nnz / kSegLen + sched_max_multi(nnz) + 1; }
size_t sched_carve(void* base, int64_t n, int64_t nnz, SchedView* view);

}  // namespace e2eg
