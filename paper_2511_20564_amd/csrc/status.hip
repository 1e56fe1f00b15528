// Status strings, the thread-local error message and the version query.
#include "common.h"

#include <vector>

namespace e2eg {

namespace {
struct Profile {
    bool active = false;
    int32_t capacity = 0;
    std::vector<hipEvent_t> start, stop;
};
thread_local Profile g_profile;
}  // namespace

void profile_mark(hipStream_t stream, bool after) {
    Profile& p = g_profile;
    if (!p.active) return;
    if (!after) {
        if ((int32_t)p.start.size() >= p.capacity) return;
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return;
        (void)hipEventRecord(e, stream);
        p.start.push_back(e);
    } else {
        if (p.stop.size() >= p.start.size()) return;
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return;
        (void)hipEventRecord(e, stream);
        p.stop.push_back(e);
    }
}

static thread_local char g_last_error[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof(g_last_error), fmt, ap);
    va_end(ap);
}

int32_t fail(int32_t status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof(g_last_error), fmt, ap);
    va_end(ap);
    return status;
}

size_t sched_carve(void* base, int64_t n, int64_t nnz, SchedView* view, bool weighted) {
    Carver c(base);
    SchedView v;
    v.max_plain = sched_max_plain(nnz);
    v.max_seg = sched_max_seg(n, nnz);
    v.max_multi = sched_max_multi(nnz);
    v.max_slot = sched_max_slot(n, nnz);
    v.header = c.take<SchedHeader>(1);
    v.orig = c.take<int32_t>(n > 0 ? n : 1);
    v.zpos = c.take<int32_t>(n > 0 ? n : 1);
    v.zrow_ptr = c.take<int32_t>(n + 1);
    v.zcol = c.take<int32_t>(nnz > 0 ? nnz : 1);
    v.short_rows = c.take<int32_t>(n > 0 ? n : 1);
    v.multi_row = c.take<int32_t>(v.max_multi);
    v.slot_base = c.take<int32_t>(v.max_multi);
    v.slot_cnt = c.take<int32_t>(v.max_multi);
    v.segs = c.take<Segment>(v.max_seg);
    v.znode = c.take<int32_t>(nnz > 0 ? nnz : 1);
    v.zs = c.take<float>(nnz > 0 ? nnz : 1);
    v.zval = weighted ? c.take<float>(nnz > 0 ? nnz : 1) : nullptr;  // last: the rest of the layout is shared
    if (view) *view = v;
    return c.size();
}

}  // namespace e2eg

namespace e2eg {
// Plain streaming copy, 16 bytes per thread: the traffic of known size against which hardware
// byte counters are scaled.
__global__ void copy_bytes16(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t chunks) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < chunks) dst[i] = src[i];
}
}  // namespace e2eg

extern "C" {

const char* e2eg_status_string(int32_t status) {
    switch (status) {
        case E2EG_OK: return "ok";
        case E2EG_ERR_INVALID_ARG: return "invalid argument";
        case E2EG_ERR_NULL_PTR: return "null pointer";
        case E2EG_ERR_BAD_DTYPE: return "unsupported dtype";
        case E2EG_ERR_CAPACITY: return "output capacity too small";
        case E2EG_ERR_OVERFLOW: return "size does not fit in int32";
        case E2EG_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case E2EG_ERR_HIP: return "HIP runtime error";
        case E2EG_ERR_BAD_INDEX: return "input id out of range";
        default: return "unknown status";
    }
}

const char* e2eg_last_error(void) { return e2eg::g_last_error; }

int32_t e2eg_version(void) { return 100; }

int32_t e2eg_profile_begin(int32_t capacity) {
    if (capacity < 0) return e2eg::fail(E2EG_ERR_INVALID_ARG, "profile_begin: negative capacity");
    e2eg::Profile& p = e2eg::g_profile;
    for (hipEvent_t e : p.start) (void)hipEventDestroy(e);
    for (hipEvent_t e : p.stop) (void)hipEventDestroy(e);
    p.start.clear();
    p.stop.clear();
    p.capacity = capacity;
    p.active = true;
    return E2EG_OK;
}

int32_t e2eg_profile_end(float* h_ms, int32_t h_capacity, int32_t* h_count) {
    e2eg::Profile& p = e2eg::g_profile;
    p.active = false;
    if (!h_count || (h_capacity > 0 && !h_ms)) return e2eg::fail(E2EG_ERR_NULL_PTR, "profile_end: null pointer");
    const int32_t count = (int32_t)(p.stop.size() < p.start.size() ? p.stop.size() : p.start.size());
    int32_t status = E2EG_OK;
    for (int32_t k = 0; k < count; ++k) {
        hipError_t err = hipEventSynchronize(p.stop[k]);
        float ms = 0.0f;
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, p.start[k], p.stop[k]);
        if (err != hipSuccess) status = e2eg::fail(E2EG_ERR_HIP, "profile_end: %s", hipGetErrorString(err));
        if (k < h_capacity) h_ms[k] = ms;
    }
    *h_count = count;
    for (hipEvent_t e : p.start) (void)hipEventDestroy(e);
    for (hipEvent_t e : p.stop) (void)hipEventDestroy(e);
    p.start.clear();
    p.stop.clear();
    return status;
}

int32_t e2eg_profile_copy(void* d_dst, const void* d_src, size_t nbytes, void* stream) {
    if (!d_dst || !d_src) return e2eg::fail(E2EG_ERR_NULL_PTR, "profile_copy: null pointer");
    if (nbytes % 16 != 0 || !e2eg::aligned_to(d_dst, 16) || !e2eg::aligned_to(d_src, 16))
        return e2eg::fail(E2EG_ERR_INVALID_ARG, "profile_copy: pointers and size must be multiples of 16 bytes");
    if (nbytes == 0) return E2EG_OK;
    const size_t chunks = nbytes / 16;
    e2eg::copy_bytes16<<<dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<uint4*>(d_dst), static_cast<const uint4*>(d_src), chunks);
    E2EG_LAUNCH_CHECK("copy_bytes16");
    return E2EG_OK;
}

}  // extern "C"
