// Optional per-launch timing with HIP events (ivit_trace_begin / ivit_trace_end in include/ivit.h).
// While a trace is active every kernel launch of the library is bracketed by two events recorded on the
// stream the kernel is launched on; ivit_trace_end synchronises the last event and reports the elapsed
// time, the kind and the algorithmic work of every launch.  Inactive, the cost is one pointer test per launch.
#include <vector>

#include "../../include/ivit.h"
#include "ivit_kernels.hpp"

namespace ivit {

namespace {
struct Trace {
    std::vector<hipEvent_t> start, stop;
    std::vector<int32_t> kind;
    std::vector<int64_t> ops, bytes;
    int count = 0;
    bool failed = false;
};
Trace* g_trace = nullptr;
}  // namespace

TraceScope::TraceScope(hipStream_t s, int kind, int64_t ops, int64_t bytes) : stream_(s), slot_(-1) {
    Trace* t = g_trace;
    if (!t) return;
    if (t->count >= (int)t->start.size()) { t->failed = true; return; }
    slot_ = t->count++;
    t->kind[slot_] = kind; t->ops[slot_] = ops; t->bytes[slot_] = bytes;
    if (hipEventRecord(t->start[slot_], s) != hipSuccess) t->failed = true;
}

TraceScope::~TraceScope() {
    Trace* t = g_trace;
    if (!t || slot_ < 0) return;
    if (hipEventRecord(t->stop[slot_], stream_) != hipSuccess) t->failed = true;
}

}  // namespace ivit

extern "C" {

int ivit_trace_begin(int32_t max_launches) {
    using namespace ivit;
    if (max_launches < 1 || max_launches > (1 << 22)) return IVIT_ERR_SHAPE;
    if (g_trace) return IVIT_ERR_PARAM;                       // a trace is already active
    Trace* t = new Trace();
    t->start.assign(max_launches, nullptr); t->stop.assign(max_launches, nullptr);
    t->kind.resize(max_launches); t->ops.resize(max_launches); t->bytes.resize(max_launches);
    bool ok = true;
    for (int i = 0; i < max_launches && ok; ++i)
        ok = hipEventCreate(&t->start[i]) == hipSuccess && hipEventCreate(&t->stop[i]) == hipSuccess;
    if (!ok) {
        for (int i = 0; i < max_launches; ++i) {
            if (t->start[i]) (void)hipEventDestroy(t->start[i]);
            if (t->stop[i]) (void)hipEventDestroy(t->stop[i]);
        }
        delete t;
        return IVIT_ERR_HIP;
    }
    g_trace = t;
    return IVIT_OK;
}

int ivit_trace_end(float* ms, int32_t* kind, int64_t* ops, int64_t* bytes, int32_t capacity, int32_t* count) {
    using namespace ivit;
    Trace* t = g_trace;
    if (!t) return IVIT_ERR_PARAM;
    g_trace = nullptr;
    int status = t->failed ? IVIT_ERR_HIP : IVIT_OK;
    const int n = t->count;
    if (count) *count = n;
    for (int i = 0; i < n && status == IVIT_OK; ++i) {
        if (hipEventSynchronize(t->stop[i]) != hipSuccess) { status = IVIT_ERR_HIP; break; }
        if (i < capacity) {
            float v = 0.f;
            if (ms && hipEventElapsedTime(&v, t->start[i], t->stop[i]) != hipSuccess) { status = IVIT_ERR_HIP; break; }
            if (ms) ms[i] = v;
            if (kind) kind[i] = t->kind[i];
            if (ops) ops[i] = t->ops[i];
            if (bytes) bytes[i] = t->bytes[i];
        }
    }
    for (size_t i = 0; i < t->start.size(); ++i) { (void)hipEventDestroy(t->start[i]); (void)hipEventDestroy(t->stop[i]); }
    delete t;
    return status;
}

}  // extern "C"
