// Status strings, the thread-local error message and the version query.
#include "common.h"

namespace e2eg {

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

size_t sched_carve(void* base, int64_t n, int64_t nnz, SchedView* view) {
    Carver c(base);
    SchedView v;
    v.max_items = sched_max_items(n, nnz);
    v.max_split = sched_max_split(nnz);
    v.header = c.take<SchedHeader>(1);
    v.item_row = c.take<int32_t>(v.max_items);
    v.item_beg = c.take<int32_t>(v.max_items);
    v.item_slot = c.take<int32_t>(v.max_items);
    v.split_row = c.take<int32_t>(v.max_split);
    v.split_base = c.take<int32_t>(v.max_split);
    v.split_cnt = c.take<int32_t>(v.max_split);
    if (view) *view = v;
    return c.size();
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

}  // extern "C"
