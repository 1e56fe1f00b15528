// e2eg_normalize: d~_i = sum_j A~_ij and d~_i^-1/2 (paper: Section 3, "Notation"), and the
// private, renumbered copy of the graph that the propagation kernels read.
//
// Renumbering.  The kTopNodes nodes of highest degree get internal ids 0, 1, ... by descending
// degree (ties in node order); all other nodes follow in node order.  The CSR is rewritten in
// internal ids, rows in internal order, columns ascending.  What this buys on a power-law
// user-item graph:
//   - the feature rows of the most popular nodes are one contiguous block, and every neighbour
//     list starts with its popular entries;
//   - everything else keeps the caller's node order (users, then items), so at any time the
//     whole GPU gathers from the same side of the graph and the L2 caches hold one hot set.
// Rows of at most kShortMax entries are listed ordered by length inside blocks of kSortBlock
// consecutive rows (the kernel sums several of them side by side, so neighbours in the list should
// be equally long, while the block-wise order keeps the users-then-items progression).  Longer
// rows are cut into segments of kSegLen entries, the very longest ones first at the boundaries
// of windows of kWindow internal ids; the segments of rows with several are ordered by first
// column, so that segments which read the same stretch of feature rows can be run at the same
// time on the same L2 (the list is dealt out to the XCDs in contiguous stretches of equal entry
// counts); rows of one segment follow in row order.
// All of it is integer work: radix sorts and scans, with sort keys only as wide as the graph
// needs, so that a small (sampled) graph costs few launches.  Nothing here depends on the feature
// width.  For a weighted graph (e2eg_normalize_weighted) d~ is the sum of the row's values and
// the values are carried into the schedule in the order of its column indices.
#include "common.h"

namespace e2eg {
namespace {

constexpr int kThreads = 256;
// The symmetry test of unpack_columns keeps a flag (asym[0]) and a count spread over kSymCounters
// addresses, one cache line each (asym[k * kSymStride], k = 1 .. kSymCounters).
constexpr int kSymCounters = 64;
constexpr int kSymStride = 32;
constexpr int kLengthCutCost = 6;   // in quarters: an entry of a segment cut by length only weighs 1.5 entries in the deal

// Per node: degree, d^-1/2, and the sort key (larger degree first, then node id): n - d in the
// upper half, which needs bits_for(n + 1) bits, so small graphs sort in few passes.
__global__ void row_stats(const int32_t* __restrict__ row_ptr, int64_t n, int32_t* __restrict__ deg,
                          float* __restrict__ dinv_sqrt, uint64_t* __restrict__ keys) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t d = row_ptr[i + 1] - row_ptr[i];
    if (deg) deg[i] = d;
    dinv_sqrt[i] = d > 0 ? (float)(1.0 / sqrt((double)d)) : 0.0f;
    keys[i] = ((uint64_t)(uint32_t)(d > n ? 0 : (int32_t)n - d) << 32) | (uint32_t)i;
}

// Sorted (degree, node) keys -> is the node one of the kTopNodes most popular, and its rank.
// Also clears the flag that unpack_columns raises for a structure that is not symmetric.
__global__ void mark_top(const uint64_t* __restrict__ sorted, int64_t n, int32_t* __restrict__ rank_of,
                         int32_t* __restrict__ not_top, int32_t* __restrict__ asym) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p > n) return;
    if (p == n) {
        not_top[p] = 0;
        for (int k = 0; k <= kSymCounters; ++k) asym[k * kSymStride] = 0;
        return;
    }
    const int32_t i = (int32_t)(uint32_t)sorted[p];
    rank_of[i] = (int32_t)p;
    not_top[i] = p < kTopNodes ? 0 : 1;
}

// Row classes by length d:  short d <= kShortMax;  plain kShortMax < d, cut by length only (one
// segment if d <= kSegLen);  wide: one of the first kMaxWide internal rows with d >= wide_min,
// cut at window boundaries first.  Rows with d > kSegLen ("multi") leave partial sums.
//
// others_before = exclusive scan of not_top over node ids.  Internal position: top nodes by
// rank, the others behind them in node order.  Also per internal row: its length, how it is cut,
// and the key that orders the short rows (block of kSortBlock rows, then length, then row).
__global__ void permute_nodes(const int32_t* __restrict__ rank_of, const int32_t* __restrict__ others_before,
                              const int32_t* __restrict__ row_ptr, int64_t n, int32_t wide_min,
                              int32_t* __restrict__ orig, int32_t* __restrict__ zpos,
                              int32_t* __restrict__ zdeg, int32_t* __restrict__ nseg,
                              int32_t* __restrict__ nslot, int32_t* __restrict__ is_short,
                              int32_t* __restrict__ is_multi, uint64_t* __restrict__ short_keys) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n) return;
    if (i == n) {  // terminators so that the scans deliver the totals at index n
        zdeg[i] = 0;
        nseg[i] = 0;
        nslot[i] = 0;
        is_short[i] = 0;
        is_multi[i] = 0;
        return;
    }
    const int32_t n_top = n < kTopNodes ? (int32_t)n : kTopNodes;
    const int32_t r = rank_of[i];
    const int32_t p = r < kTopNodes ? r : n_top + others_before[i];
    const int32_t d = row_ptr[i + 1] - row_ptr[i];
    const int32_t segs = (d + kSegLen - 1) / kSegLen;
    const bool wide = p < kMaxWide && d >= wide_min;
    orig[p] = (int32_t)i;
    zpos[i] = p;
    zdeg[p] = d;
    nseg[p] = (d > kShortMax && !wide) ? segs : 0;   // segments made by cutting by length
    nslot[p] = (d > kSegLen && !wide) ? segs : 0;    // those of them that are partial-sum slots
    is_short[p] = d <= kShortMax ? 1 : 0;
    is_multi[p] = d > kSegLen ? 1 : 0;
    // longer rows sort behind every short one: one block number past the last
    const uint32_t hi = d > kShortMax ? ((uint32_t)(n / kSortBlock) + 1u) << 8 : (((uint32_t)p / kSortBlock) << 8) | (uint32_t)d;
    short_keys[p] = ((uint64_t)hi << 32) | (uint32_t)p;
}

// Wide rows, one thread per (row p, window boundary w), w = 0 .. nwin: position of the first entry
// of row p with column >= w * kWindow.  Rows that are not wide get an empty range everywhere.
__global__ void wide_bounds(SchedView s, int32_t wide_rows, int32_t nwin, int32_t wide_min,
                            int32_t* __restrict__ bounds) {
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (int64_t)wide_rows * (nwin + 1)) return;
    const int32_t p = (int32_t)(id / (nwin + 1));
    const int32_t w = (int32_t)(id - (int64_t)p * (nwin + 1));
    const int32_t beg = s.zrow_ptr[p], end = s.zrow_ptr[p + 1];
    if (end - beg < wide_min) {
        bounds[id] = beg;
        return;
    }
    const int64_t key = (int64_t)w * kWindow;
    int32_t lo = beg, hi = end;  // first position with zcol >= key
    while (lo < hi) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        if (s.zcol[mid] < key) lo = mid + 1; else hi = mid;
    }
    bounds[id] = lo;
}

// One thread per (wide row, window): segments needed for its run of entries.
__global__ void wide_counts(int32_t wide_rows, int32_t nwin, const int32_t* __restrict__ bounds,
                            int32_t* __restrict__ pair_nseg) {
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t pairs = (int64_t)wide_rows * nwin;
    if (id > pairs) return;
    if (id == pairs) {
        pair_nseg[id] = 0;
        return;
    }
    const int32_t p = (int32_t)(id / nwin);
    const int32_t w = (int32_t)(id - (int64_t)p * nwin);
    const int32_t cnt = bounds[(int64_t)p * (nwin + 1) + w + 1] - bounds[(int64_t)p * (nwin + 1) + w];
    pair_nseg[id] = (cnt + kSegLen - 1) / kSegLen;
}

struct RowScans {          // exclusive scans over internal rows, n + 1 entries each
    const int32_t* seg_off;
    const int32_t* slot_off;
    const int32_t* short_off;
    const int32_t* multi_off;
};

// Header and the list of rows that leave partial sums.  pair_off = exclusive scan of pair_nseg.
__global__ void emit_rows(RowScans sc, const int32_t* __restrict__ pair_off, int32_t wide_rows, int32_t nwin,
                          int32_t wide_min, int64_t n, int64_t nnz, const int32_t* __restrict__ asym, SchedView s) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p > n) return;
    const int32_t n_slot_plain = sc.slot_off[n];
    const int32_t n_wide_slots = wide_rows > 0 ? pair_off[(int64_t)wide_rows * nwin] : 0;
    if (p == n) {
        SchedHeader h;
        h.n_short = sc.short_off[n];
        h.n_seg = sc.seg_off[n] + n_wide_slots;
        h.n_slot = n_slot_plain + n_wide_slots;
        h.n_multi = sc.multi_off[n];
        h.n = (int32_t)n;
        h.nnz = (int32_t)nnz;
        uint32_t balance = 0;   // looking minus not-looking entries (see unpack_columns), modulo 2^32
        for (int k = 1; k <= kSymCounters; ++k) balance += (uint32_t)asym[k * kSymStride];
        h.flags = (asym[0] != 0 || balance != 0) ? kSchedNotSymmetric : 0;
        h.pad = 0;
        for (int x = 0; x <= kXcds; ++x) h.xcd_first[x] = h.n_slot;  // lowered by deal_segments
        for (int x = 0; x < 7; ++x) h.pad2[x] = 0;
        *s.header = h;
        return;
    }
    const int32_t d = s.zrow_ptr[p + 1] - s.zrow_ptr[p];
    if (d > kSegLen) {
        const int32_t m = sc.multi_off[p];
        s.multi_row[m] = (int32_t)p;
        if (p < wide_rows && d >= wide_min) {
            s.slot_base[m] = n_slot_plain + pair_off[(int64_t)p * nwin];
            s.slot_cnt[m] = pair_off[(int64_t)(p + 1) * nwin] - pair_off[(int64_t)p * nwin];
        } else {
            s.slot_base[m] = sc.slot_off[p];
            s.slot_cnt[m] = (d + kSegLen - 1) / kSegLen;
        }
    }
}

// Sort key of a segment (upper half; the lower half is the segment's number t, which is also its
// place in the key array, so the stable sort keeps equal keys in order of t): slotted segments by
// first column, then the one-segment rows, which all carry 2^bits with bits = bits_for(n).
__device__ __forceinline__ uint64_t segment_key(const SchedView& s, const Segment& g, int32_t t, int bits) {
    const uint32_t hi = g.slot >= 0 ? (uint32_t)s.zcol[g.beg] : 1u << bits;
    return ((uint64_t)hi << 32) | (uint32_t)t;
}

// Segments of rows cut by length only.  One thread per segment t: find its row (binary search in
// seg_off, the ascending first segment number of every row; rows without such segments repeat
// their successor's number and are skipped by taking the last row whose number is <= t).
__global__ void emit_plain_segments(SchedView s, RowScans sc, int64_t n, int bits, Segment* __restrict__ seg_tmp,
                                    uint64_t* __restrict__ keys) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= sc.seg_off[n]) return;
    int64_t lo = 0, hi = n - 1;  // last p with seg_off[p] <= t
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (sc.seg_off[mid] <= t) lo = mid; else hi = mid - 1;
    }
    const int32_t row = (int32_t)lo;
    const int32_t q = (int32_t)t - sc.seg_off[row];
    const int32_t row_beg = s.zrow_ptr[row], row_end = s.zrow_ptr[row + 1];
    const int32_t beg = row_beg + q * kSegLen;
    const int32_t end = beg + kSegLen < row_end ? beg + kSegLen : row_end;
    const Segment g{row, beg, end, row_end - row_beg > kSegLen ? sc.slot_off[row] + q : -1};
    seg_tmp[t] = g;
    keys[t] = segment_key(s, g, (int32_t)t, bits);
}

// Segments of wide rows: one thread per (row, window) cuts that run by length.
__global__ void emit_wide_segments(SchedView s, RowScans sc, int64_t n, int bits, int32_t wide_rows, int32_t nwin,
                                   const int32_t* __restrict__ bounds, const int32_t* __restrict__ pair_off,
                                   Segment* __restrict__ seg_tmp, uint64_t* __restrict__ keys) {
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (int64_t)wide_rows * nwin) return;
    const int32_t p = (int32_t)(id / nwin);
    const int32_t w = (int32_t)(id - (int64_t)p * nwin);
    const int32_t run_beg = bounds[(int64_t)p * (nwin + 1) + w], run_end = bounds[(int64_t)p * (nwin + 1) + w + 1];
    const int32_t t0 = sc.seg_off[n] + pair_off[id];        // behind the plain segments
    const int32_t slot0 = sc.slot_off[n] + pair_off[id];    // behind the plain slots
    int32_t q = 0;
    for (int32_t beg = run_beg; beg < run_end; beg += kSegLen, ++q) {
        const Segment g{p, beg, beg + kSegLen < run_end ? beg + kSegLen : run_end, slot0 + q};
        seg_tmp[t0 + q] = g;
        keys[t0 + q] = segment_key(s, g, t0 + q, bits);
    }
}

__global__ void fill_keys(uint64_t* __restrict__ keys, int64_t count) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < count) keys[k] = ~0ull;  // sorts behind every real segment
}

// Sorted keys -> the ordered segment list, and each slotted segment's length for the deal.
// (A segment cut by length only reaches across many windows and mostly misses in L2, so its
// entries count kLengthCutCost / 4 times in the deal; such segments have the lowest first columns
// and would otherwise make the first XCD's stretch the slowest.)
__global__ void place_segments(const uint64_t* __restrict__ keys, const Segment* __restrict__ seg_tmp,
                               SchedView s, int32_t wide_rows, int32_t wide_min, uint64_t* __restrict__ seg_len) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p > s.max_seg) return;
    uint64_t len = 0;
    if (p < s.header->n_seg) {
        const Segment g = seg_tmp[(uint32_t)keys[p]];
        s.segs[p] = g;
        if (p < s.header->n_slot) {
            const bool wide = g.row < wide_rows && s.zrow_ptr[g.row + 1] - s.zrow_ptr[g.row] >= wide_min;
            len = wide ? (uint64_t)(g.end - g.beg) : (uint64_t)(g.end - g.beg) * kLengthCutCost / 4;
        }
    }
    seg_len[p] = len;
}

// len_off = exclusive scan of seg_len (max_seg + 1 entries; the last is the total; 64-bit, since
// the weighted counts of a graph near the int32 limit of nnz pass 2^31).  XCD x gets the slotted
// segments whose running entry count starts in [x, x+1) eighths of the total.
__global__ void deal_segments(const uint64_t* __restrict__ len_off, SchedView s) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int32_t n_slot = s.header->n_slot;
    if (p >= n_slot) return;
    const int64_t total = (int64_t)len_off[s.max_seg];
    const int64_t here = (int64_t)len_off[p], prev = p > 0 ? (int64_t)len_off[p - 1] : -1;
    for (int x = 0; x < kXcds; ++x) {
        const int64_t mark = total * x / kXcds;   // first segment whose start count is >= mark
        if (here >= mark && prev < mark) s.header->xcd_first[x] = (int32_t)p;
    }
}

__global__ void place_short_rows(const uint64_t* __restrict__ keys, int64_t n, SchedView s) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < n) s.short_rows[k] = (int32_t)(uint32_t)keys[k];  // the first n_short are the short rows
}

// One thread per CSR entry e: key = (internal row << bits) | internal column.
// The row of entry e: the last i in [lo, hi] with row_ptr[i] <= e.
__device__ __forceinline__ int64_t row_of_entry(const int32_t* __restrict__ row_ptr, int64_t e, int64_t lo, int64_t hi) {
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (row_ptr[mid] <= e) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// A workgroup's entries are consecutive, so their rows lie between the rows of its first and of
// its last entry: two threads search all rows for those, the others then search that short range.
__global__ __launch_bounds__(kThreads) void entry_keys(const int32_t* __restrict__ row_ptr,
                                                       const int32_t* __restrict__ col_idx,
                                                       const int32_t* __restrict__ zpos, int64_t n, int64_t nnz,
                                                       int bits, uint64_t* __restrict__ keys) {
    __shared__ int64_t range[2];
    const int64_t first = (int64_t)blockIdx.x * kThreads;
    const int64_t e = first + threadIdx.x;
    if (threadIdx.x == 0) range[0] = row_of_entry(row_ptr, first, 0, n - 1);
    if (threadIdx.x == 64) {
        const int64_t last = first + kThreads - 1 < nnz ? first + kThreads - 1 : nnz - 1;
        range[1] = row_of_entry(row_ptr, last, 0, n - 1);
    }
    __syncthreads();
    if (e >= nnz) return;
    const int64_t row = row_of_entry(row_ptr, e, range[0], range[1]);
    keys[e] = ((uint64_t)(uint32_t)zpos[row] << bits) | (uint32_t)zpos[col_idx[e]];
}

// Sorted (row, column) keys -> the column array.  The same pass decides whether the structure is
// symmetric (the transposed entry points run on this schedule only if it is).  Of the two entries of
// a symmetric pair exactly one "looks": the one whose own row is the longer (ties: the larger row id).
// It searches for its mirror (column, row) in the other row's stretch of the sorted keys, which is
// the shorter one, so no search walks a popular node's row.  The structure is symmetric iff every
// looking entry finds its mirror and there are as many looking as not-looking entries (the mirrors
// found are distinct not-looking entries; equal counts leave none without a partner).
__global__ __launch_bounds__(kThreads) void unpack_columns(const uint64_t* __restrict__ keys, int64_t nnz, int bits,
                                                           const int32_t* __restrict__ zrow_ptr,
                                                           int32_t* __restrict__ zcol, int32_t* __restrict__ asym) {
    __shared__ int32_t balance;
    if (threadIdx.x == 0) balance = 0;
    __syncthreads();
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int32_t mine = 0;   // +1 looking, -1 not looking, 0 diagonal / past the end
    if (e < nnz) {
        const uint64_t key = keys[e];
        const uint32_t c = (uint32_t)(key & ((1ull << bits) - 1));
        const uint32_t r = (uint32_t)(key >> bits);
        zcol[e] = (int32_t)c;
        if (r != c) {
            const int32_t cb = zrow_ptr[c], ce = zrow_ptr[c + 1];
            const int32_t own = zrow_ptr[r + 1] - zrow_ptr[r], other = ce - cb;
            const bool looks = own > other || (own == other && r > c);
            mine = looks ? 1 : -1;
            if (looks) {
                const uint64_t mirror = ((uint64_t)c << bits) | r;
                int32_t lo = cb, hi = ce;   // first position with key >= mirror
                while (lo < hi) {
                    const int32_t mid = lo + ((hi - lo) >> 1);
                    if (keys[mid] < mirror) lo = mid + 1; else hi = mid;
                }
                if (lo >= ce || keys[lo] != mirror) atomicOr(asym, 1);
            }
        }
    }
    for (int off = 32; off > 0; off >>= 1) mine += __shfl_down(mine, off);
    if ((threadIdx.x & 63) == 0 && mine != 0) atomicAdd(&balance, mine);
    __syncthreads();
    if (threadIdx.x == 0 && balance != 0)
        atomicAdd(asym + (1 + blockIdx.x % kSymCounters) * kSymStride, balance);
}

// Weighted graphs.  d~_i = sum of the stored values of row i (the diagonal entry carries the 1 of
// D~ = D + I); one wavefront per row, lanes stride over the row, lane sums added in lane order.
__global__ __launch_bounds__(kThreads) void weighted_degrees(const int32_t* __restrict__ row_ptr,
                                                             const float* __restrict__ val, int64_t n,
                                                             float* __restrict__ deg_w,
                                                             float* __restrict__ dinv_sqrt) {
    const int lane = threadIdx.x & 63;
    const int64_t row = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6;
    if (row >= n) return;
    const int32_t beg = row_ptr[row], end = row_ptr[row + 1];
    double s = 0.0;
    for (int32_t p = beg + lane; p < end; p += 64) s += (double)val[p];
    for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off);   // fixed tree
    if (lane == 0) {
        if (deg_w) deg_w[row] = (float)s;
        dinv_sqrt[row] = s > 0.0 ? (float)(1.0 / sqrt(s)) : 0.0f;
    }
}

// One thread per stored entry e of the caller's CSR: its value goes to the place of the same entry
// in the internal CSR (row zpos[i], column zpos[j], found by binary search in that row).
__global__ __launch_bounds__(kThreads) void place_values(const int32_t* __restrict__ row_ptr,
                                                         const int32_t* __restrict__ col_idx,
                                                         const float* __restrict__ val, int64_t n, int64_t nnz,
                                                         SchedView s) {
    __shared__ int64_t range[2];   // rows of the workgroup's first and last entry (see entry_keys)
    const int64_t first = (int64_t)blockIdx.x * kThreads;
    const int64_t e = first + threadIdx.x;
    if (threadIdx.x == 0) range[0] = row_of_entry(row_ptr, first, 0, n - 1);
    if (threadIdx.x == 64) {
        const int64_t last = first + kThreads - 1 < nnz ? first + kThreads - 1 : nnz - 1;
        range[1] = row_of_entry(row_ptr, last, 0, n - 1);
    }
    __syncthreads();
    if (e >= nnz) return;
    const int64_t lo = row_of_entry(row_ptr, e, range[0], range[1]);
    const int32_t p = s.zpos[lo];
    const int32_t c = s.zpos[col_idx[e]];
    int32_t a = s.zrow_ptr[p], b = s.zrow_ptr[p + 1];   // first position with zcol >= c
    while (a < b) {
        const int32_t mid = a + ((b - a) >> 1);
        if (s.zcol[mid] < c) a = mid + 1; else b = mid;
    }
    if (a < s.zrow_ptr[p + 1] && s.zcol[a] == c) s.zval[a] = val[e];
    // the mirror entry (j, i) of the caller's CSR must carry the same value (bit for bit), or the
    // transposed entry points would apply another operator than the transpose
    const int32_t j = col_idx[e];
    if (j == (int32_t)lo) return;
    int32_t ma = row_ptr[j], mb = row_ptr[j + 1];   // first position in row j with column >= i
    const int32_t mend = mb;
    while (ma < mb) {
        const int32_t mid = ma + ((mb - ma) >> 1);
        if (col_idx[mid] < (int32_t)lo) ma = mid + 1; else mb = mid;
    }
    if (ma >= mend || col_idx[ma] != (int32_t)lo || __float_as_uint(val[ma]) != __float_as_uint(val[e]))
        atomicOr(&s.header->flags, kSchedValuesNotSymmetric);
}

// One thread per entry of the internal CSR: its column as a node id and that node's d~^-1/2 (times
// the entry's value on a weighted graph).  The first layer of a propagation reads these beside each
// other and gathers the caller's feature rows directly, which saves the pass that would pre-scale them.
__global__ void entry_scales(SchedView s, const float* __restrict__ dinv_sqrt, int64_t nnz) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= nnz) return;
    const int32_t node = s.orig[s.zcol[e]];
    s.znode[e] = node;
    s.zs[e] = s.zval ? s.zval[e] * dinv_sqrt[node] : dinv_sqrt[node];
}

__global__ void zero_values(float* __restrict__ v, int64_t count) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < count) v[e] = 0.0f;
}

struct NormWs {
    uint64_t* keys_a;
    uint64_t* keys_b;
    int32_t* rank_of;
    int32_t* not_top;
    int32_t* zdeg;
    int32_t* nseg;
    int32_t* nslot;
    int32_t* is_short;
    int32_t* is_multi;
    int32_t* bounds;     // [wide rows][windows + 1]
    int32_t* pair_nseg;  // [wide rows * windows + 1]
    uint64_t* seg_len;   // [max_seg + 1]
    int32_t* asym;       // symmetry flag and spread counters (see unpack_columns)
    Segment* seg_tmp;
    void* scan_ws;
    void* sort_ws;
    size_t bytes;
};

NormWs carve_norm(void* base, int64_t n, int64_t nnz) {
    Carver c(base);
    NormWs w;
    const int64_t max_seg = sched_max_seg(n, nnz);
    int64_t m = n + 1 > nnz ? n + 1 : nnz;
    if (max_seg + 1 > m) m = max_seg + 1;
    w.keys_a = c.take<uint64_t>(m);
    w.keys_b = c.take<uint64_t>(m);
    w.rank_of = c.take<int32_t>(n + 1);
    w.not_top = c.take<int32_t>(n + 1);
    w.zdeg = c.take<int32_t>(n + 1);
    w.nseg = c.take<int32_t>(n + 1);
    w.nslot = c.take<int32_t>(n + 1);
    w.is_short = c.take<int32_t>(n + 1);
    w.is_multi = c.take<int32_t>(n + 1);
    w.bounds = c.take<int32_t>(sched_max_wide_rows(n) * (sched_windows(n) + 1) + 1);
    w.pair_nseg = c.take<int32_t>(sched_max_pairs(n) + 1);
    w.seg_len = c.take<uint64_t>(max_seg + 1);
    w.asym = c.take<int32_t>((kSymCounters + 1) * kSymStride);
    w.seg_tmp = c.take<Segment>(max_seg);
    w.scan_ws = c.take<char>(5 * scan_workspace_bytes(m));   // the five row scans share one set of launches
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

extern "C" size_t e2eg_sched_weighted_bytes(int32_t n, int64_t nnz) {
    if (n < 0 || nnz < 0) return 0;
    return sched_carve(nullptr, n, nnz, nullptr, true);
}

extern "C" size_t e2eg_normalize_workspace_bytes(int32_t n, int64_t nnz) {
    if (n < 0 || nnz < 0) return 0;
    return carve_norm(nullptr, n, nnz).bytes;
}

namespace {
// d_val == nullptr: the unweighted call.  Otherwise d~ and d~^-1/2 come from the values (d_deg_w may
// be null), d_deg receives the row lengths, and the schedule also receives the values in internal order.
int32_t normalize_impl(int32_t n, int64_t nnz, const int32_t* d_row_ptr, const int32_t* d_col_idx,
                       const float* d_val, int32_t* d_deg, float* d_deg_w, float* d_dinv_sqrt, void* d_sched,
                       size_t sched_bytes, void* ws, size_t ws_bytes, void* stream_) {
    const bool weighted = d_val != nullptr;
    if (n < 0 || nnz < 0) return fail(E2EG_ERR_INVALID_ARG, "normalize: negative size");
    if (nnz > (int64_t)INT32_MAX || n == INT32_MAX)
        return fail(E2EG_ERR_OVERFLOW, "normalize: nnz=%lld exceeds int32", (long long)nnz);
    if (!d_row_ptr || !d_dinv_sqrt || !d_sched || (nnz > 0 && !d_col_idx))
        return fail(E2EG_ERR_NULL_PTR, "normalize: null pointer");
    const size_t sched_need = sched_carve(nullptr, n, nnz, nullptr, weighted);
    if (!aligned_to(d_sched, kAlign) || sched_bytes < sched_need)
        return fail(E2EG_ERR_CAPACITY, "normalize: d_sched needs %zu bytes, 256-byte aligned", sched_need);
    const size_t need = e2eg_normalize_workspace_bytes(n, nnz);
    if (!ws || !aligned_to(ws, kAlign) || ws_bytes < need)
        return fail(E2EG_ERR_WORKSPACE, "normalize: workspace needs %zu bytes, 256-byte aligned", need);

    hipStream_t stream = static_cast<hipStream_t>(stream_);
    NormWs w = carve_norm(ws, n, nnz);
    SchedView view;
    sched_carve(d_sched, n, nnz, &view, weighted);
    const dim3 blk(kThreads);

    // 1. degrees, d^-1/2, popularity order, internal numbering
    uint64_t* src = w.keys_a;
    uint64_t* dst = w.keys_b;
    if (n > 0) {
        row_stats<<<grid_for(n), blk, 0, stream>>>(d_row_ptr, n, d_deg, d_dinv_sqrt, src);
        E2EG_LAUNCH_CHECK("row_stats");
        int32_t st = radix_sort_u64(&src, &dst, n, 32, bits_for((int64_t)n + 1), w.sort_ws, stream);
        if (st != E2EG_OK) return st;
    }
    mark_top<<<grid_for((int64_t)n + 1), blk, 0, stream>>>(src, n, w.rank_of, w.not_top, w.asym);
    E2EG_LAUNCH_CHECK("mark_top");
    E2EG_HIP_TRY(exclusive_scan_i32(w.not_top, w.not_top, (int64_t)n + 1, nullptr, w.scan_ws, stream));
    src = w.keys_a;
    dst = w.keys_b;
    const int32_t wide_min = (int32_t)sched_wide_threshold(n);
    const int32_t wide_rows = (int32_t)sched_max_wide_rows(n);
    const int32_t nwin = (int32_t)sched_windows(n);
    permute_nodes<<<grid_for((int64_t)n + 1), blk, 0, stream>>>(w.rank_of, w.not_top, d_row_ptr, n, wide_min,
                                                               view.orig, view.zpos, w.zdeg, w.nseg, w.nslot,
                                                               w.is_short, w.is_multi, src);
    E2EG_LAUNCH_CHECK("permute_nodes");
    if (n > 0) {  // short rows: by block of kSortBlock rows, then by length
        int32_t st = radix_sort_u64(&src, &dst, n, 32, 8 + bits_for(n / kSortBlock + 2), w.sort_ws, stream);
        if (st != E2EG_OK) return st;
        place_short_rows<<<grid_for(n), blk, 0, stream>>>(src, n, view);
        E2EG_LAUNCH_CHECK("place_short_rows");
    }
    {  // five prefix sums over the internal rows, one set of launches
        const int32_t* const in[5] = {w.zdeg, w.nseg, w.nslot, w.is_short, w.is_multi};
        int32_t* const out[5] = {view.zrow_ptr, w.nseg, w.nslot, w.is_short, w.is_multi};
        E2EG_HIP_TRY(exclusive_scan_i32_batch(in, out, 5, (int64_t)n + 1, w.scan_ws, stream));
    }

    // 2. the CSR in internal ids
    if (nnz > 0) {
        const int bits = bits_for(n);
        src = w.keys_a;
        dst = w.keys_b;
        entry_keys<<<grid_for(nnz), blk, 0, stream>>>(d_row_ptr, d_col_idx, view.zpos, n, nnz, bits, src);
        E2EG_LAUNCH_CHECK("entry_keys");
        int32_t st = radix_sort_u64(&src, &dst, nnz, 0, 2 * bits, w.sort_ws, stream);
        if (st != E2EG_OK) return st;
        unpack_columns<<<grid_for(nnz), blk, 0, stream>>>(src, nnz, bits, view.zrow_ptr, view.zcol, w.asym);
        E2EG_LAUNCH_CHECK("unpack_columns");
    }

    // 3. segments: wide rows by window then length, the other long rows by length; ordered and dealt
    const RowScans sc{w.nseg, w.nslot, w.is_short, w.is_multi};
    const int64_t pairs = (int64_t)wide_rows * nwin;
    if (pairs > 0) {
        wide_bounds<<<grid_for((int64_t)wide_rows * (nwin + 1)), blk, 0, stream>>>(view, wide_rows, nwin, wide_min,
                                                                                  w.bounds);
        E2EG_LAUNCH_CHECK("wide_bounds");
        wide_counts<<<grid_for(pairs + 1), blk, 0, stream>>>(wide_rows, nwin, w.bounds, w.pair_nseg);
        E2EG_LAUNCH_CHECK("wide_counts");
        E2EG_HIP_TRY(exclusive_scan_i32(w.pair_nseg, w.pair_nseg, pairs + 1, nullptr, w.scan_ws, stream));
    }
    emit_rows<<<grid_for((int64_t)n + 1), blk, 0, stream>>>(sc, w.pair_nseg, wide_rows, nwin, wide_min, n, nnz, w.asym, view);
    E2EG_LAUNCH_CHECK("emit_rows");
    if (nnz > kShortMax) {  // otherwise no row can be long
        src = w.keys_a;
        dst = w.keys_b;
        fill_keys<<<grid_for(view.max_seg), blk, 0, stream>>>(src, view.max_seg);
        E2EG_LAUNCH_CHECK("fill_keys");
        const int bits = bits_for(n);  // columns are below 2^bits; 2^bits marks one-segment rows, all ones padding
        emit_plain_segments<<<grid_for(view.max_seg), blk, 0, stream>>>(view, sc, n, bits, w.seg_tmp, src);
        E2EG_LAUNCH_CHECK("emit_plain_segments");
        if (pairs > 0) {
            emit_wide_segments<<<grid_for(pairs), blk, 0, stream>>>(view, sc, n, bits, wide_rows, nwin, w.bounds,
                                                                   w.pair_nseg, w.seg_tmp, src);
            E2EG_LAUNCH_CHECK("emit_wide_segments");
        }
        int32_t st = radix_sort_u64(&src, &dst, view.max_seg, 32, bits + 2 < 32 ? bits + 2 : 32, w.sort_ws, stream);
        if (st != E2EG_OK) return st;
        place_segments<<<grid_for(view.max_seg + 1), blk, 0, stream>>>(src, w.seg_tmp, view, wide_rows, wide_min, w.seg_len);
        E2EG_LAUNCH_CHECK("place_segments");
        E2EG_HIP_TRY(exclusive_scan_u64(w.seg_len, w.seg_len, view.max_seg + 1, nullptr, w.scan_ws, stream));
        deal_segments<<<grid_for(view.max_slot + 1), blk, 0, stream>>>(w.seg_len, view);
        E2EG_LAUNCH_CHECK("deal_segments");
    }
    // 4. weighted graphs: d~ from the values, and the values in internal order
    if (weighted) {
        if (n > 0) {
            weighted_degrees<<<grid_for((int64_t)n * 64), blk, 0, stream>>>(d_row_ptr, d_val, n, d_deg_w, d_dinv_sqrt);
            E2EG_LAUNCH_CHECK("weighted_degrees");
        }
        if (nnz > 0) {
            // a row that lists a column twice leaves the extra places at zero (see the header)
            zero_values<<<grid_for(nnz), blk, 0, stream>>>(view.zval, nnz);
            E2EG_LAUNCH_CHECK("zero_values");
            place_values<<<grid_for(nnz), blk, 0, stream>>>(d_row_ptr, d_col_idx, d_val, n, nnz, view);
            E2EG_LAUNCH_CHECK("place_values");
        }
    }
    // 5. per entry: column as a node id, and the scale the first layer multiplies its row by
    if (nnz > 0) {
        entry_scales<<<grid_for(nnz), blk, 0, stream>>>(view, d_dinv_sqrt, nnz);
        E2EG_LAUNCH_CHECK("entry_scales");
    }
    return E2EG_OK;
}
}  // namespace

extern "C" int32_t e2eg_normalize(int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                                  const int32_t* d_col_idx, int32_t* d_deg, float* d_dinv_sqrt,
                                  void* d_sched, size_t sched_bytes, void* ws, size_t ws_bytes,
                                  void* stream) {
    return normalize_impl(n, nnz, d_row_ptr, d_col_idx, nullptr, d_deg, nullptr, d_dinv_sqrt, d_sched, sched_bytes, ws,
                          ws_bytes, stream);
}

extern "C" int32_t e2eg_normalize_weighted(int32_t n, int64_t nnz, const int32_t* d_row_ptr,
                                           const int32_t* d_col_idx, const float* d_val, int32_t* d_deg,
                                           float* d_deg_w, float* d_dinv_sqrt, void* d_sched, size_t sched_bytes,
                                           void* ws, size_t ws_bytes, void* stream) {
    if (!d_val && nnz > 0) return fail(E2EG_ERR_NULL_PTR, "normalize_weighted: d_val is null");
    static const float kOne = 1.0f;  // nnz == 0: any non-null pointer selects the weighted layout
    return normalize_impl(n, nnz, d_row_ptr, d_col_idx, d_val ? d_val : &kOne, d_deg, d_deg_w, d_dinv_sqrt, d_sched,
                          sched_bytes, ws, ws_bytes, stream);
}

extern "C" int32_t e2eg_sched_check_symmetric(const void* d_sched, void* stream_) {
    if (!d_sched) return fail(E2EG_ERR_NULL_PTR, "sched_check_symmetric: d_sched is null");
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    SchedHeader h;   // the schedule starts with its header
    E2EG_HIP_TRY(hipMemcpyAsync(&h, d_sched, sizeof(h), hipMemcpyDeviceToHost, stream));
    E2EG_HIP_TRY(hipStreamSynchronize(stream));
    if (h.flags & kSchedNotSymmetric)
        return fail(E2EG_ERR_INVALID_ARG, "sched_check_symmetric: the structure holds an entry (i, j) without (j, i); "
                                          "the transposed entry points cannot run on it");
    if (h.flags & kSchedValuesNotSymmetric)
        return fail(E2EG_ERR_INVALID_ARG, "sched_check_symmetric: the values of (i, j) and (j, i) differ somewhere; "
                                          "the transposed entry points cannot run on it");
    return E2EG_OK;
}
