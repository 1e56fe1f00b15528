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
// Up to 8 arrays of `count` values each in one set of launches (in[y] == out[y] allowed); `ws` needs
// k * scan_workspace_bytes(count).
hipError_t exclusive_scan_i32_batch(const int32_t* const* in, int32_t* const* out, int k, int64_t count, void* ws,
                                    hipStream_t stream);
// The same over uint64 (sums must stay below 2^64); `ws` needs scan_u64_workspace_bytes(count).
size_t scan_u64_workspace_bytes(int64_t count);
hipError_t exclusive_scan_u64(const uint64_t* in, uint64_t* out, int64_t count, uint64_t* d_total,
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
constexpr int kHotBytes = 128 * 1024;
constexpr int kTopNodes = kHotBytes / 16;  // nodes renumbered to the front, by descending degree
// The longest rows ("wide": among the first kMaxWide internal rows, and at least
// kWideFactor entries per window on average) are cut at the boundaries of windows of kWindow
// consecutive internal ids before they are cut by length: a segment then reads feature rows of
// one window only, and segments of the same window, run together, share them in L2.
constexpr int kWindow = 8192;
constexpr int kMaxWide = 1024;
constexpr int kWideFactor = 16;
constexpr int kXcds = 8;

struct alignas(16) Segment {
    int32_t row;   // internal row
    int32_t beg;   // first entry in zcol
    int32_t end;   // one past the last entry
    int32_t slot;  // partial-sum slot, or -1 when the segment is the whole row
};

struct SchedHeader {
    int32_t n_short;   // rows with at most kShortMax entries
    int32_t n_seg;     // all segments
    int32_t n_slot;    // segments of rows cut into several = partial-sum slots = the first n_slot of `segs`
    int32_t n_multi;   // rows cut into several segments
    int32_t n;
    int32_t nnz;
    int32_t flags;     // kSchedNotSymmetric | kSchedValuesNotSymmetric, found while the schedule was built
    int32_t pad;
    int32_t xcd_first[kXcds + 1];  // the slotted segments dealt out by equal entry counts: XCD x
                                   // owns segs[xcd_first[x] .. xcd_first[x + 1])
    int32_t pad2[7];
};

// header.flags: the stored structure holds an entry (i, j) without (j, i); the values of a weighted
// graph differ between (i, j) and (j, i).  Either makes the transposed entry points refuse the schedule.
constexpr int32_t kSchedNotSymmetric = 1;
constexpr int32_t kSchedValuesNotSymmetric = 2;

struct SchedView {
    SchedHeader* header;
    int32_t* orig;        // [n] node at internal position p
    int32_t* zpos;        // [n] internal position of node i
    int32_t* zrow_ptr;    // [n + 1] row pointers of the internal CSR
    int32_t* zcol;        // [nnz] internal column ids, ascending within each row
    int32_t* short_rows;  // [n] internal rows with at most kShortMax entries, processing order
    int32_t* multi_row;   // [max_multi] internal rows cut into several segments, ascending
    int32_t* slot_base;   // [max_multi] first slot of each such row
    int32_t* slot_cnt;    // [max_multi] number of slots
    Segment* segs;        // [max_seg]: slotted segments ordered by first column, then one-segment rows
    float* zval;          // [nnz] entry values in zcol order (weighted schedules only, else null)
    int32_t* znode;       // [nnz] orig[zcol[e]]: the column of entry e as a node id
    float* zs;            // [nnz] d~^-1/2 of that node (times the entry's value on a weighted graph)
    int64_t max_plain, max_seg, max_multi, max_slot;
};

// Upper bounds that depend on (n, nnz) only, so that launches need no device read-back.
inline int64_t sched_windows(int64_t n) { return (n + kWindow - 1) / kWindow; }
inline int64_t sched_wide_threshold(int64_t n) {
    const int64_t t = (int64_t)kWideFactor * sched_windows(n);
    return t > kSegLen ? t : kSegLen + 1;
}
inline int64_t sched_max_wide_rows(int64_t n) { return n < kMaxWide ? n : kMaxWide; }
inline int64_t sched_max_pairs(int64_t n) { return sched_max_wide_rows(n) * sched_windows(n); }
inline int64_t sched_max_plain(int64_t nnz) { return nnz / (kShortMax + 1) + 1; }  // rows cut by length only
inline int64_t sched_max_multi(int64_t nnz) { return nnz / (kSegLen + 1) + 1; }
inline int64_t sched_max_slot(int64_t n, int64_t nnz) {
    return nnz / kSegLen + sched_max_multi(nnz) + sched_max_pairs(n) + 1;
}
inline int64_t sched_max_seg(int64_t n, int64_t nnz) { return sched_max_slot(n, nnz) + sched_max_plain(nnz); }
size_t sched_carve(void* base, int64_t n, int64_t nnz, SchedView* view, bool weighted = false);

}  // namespace e2eg
