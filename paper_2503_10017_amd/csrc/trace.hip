// Measurement aid behind fnn_trace_begin / fnn_trace_end (see include/fnn_measure.h).
#include "trace.hpp"

#include <vector>

#include "../../include/fnn_measure.h"

namespace fnn {

namespace {
struct TraceState {
    bool open = false;
    int used = 0;
    std::vector<hipEvent_t> start, stop;
    std::vector<int> kind, detail;
};
TraceState g_trace;
}  // namespace

bool trace_next(int kind, int detail, hipEvent_t* start, hipEvent_t* stop) {
    if (!g_trace.open || g_trace.used >= (int)g_trace.start.size()) return false;
    *start = g_trace.start[g_trace.used];
    *stop = g_trace.stop[g_trace.used];
    g_trace.kind[g_trace.used] = kind;
    g_trace.detail[g_trace.used] = detail;
    ++g_trace.used;
    return true;
}

static void trace_release() {
    for (hipEvent_t e : g_trace.start) (void)hipEventDestroy(e);
    for (hipEvent_t e : g_trace.stop) (void)hipEventDestroy(e);
    g_trace.start.clear();
    g_trace.stop.clear();
    g_trace.kind.clear();
    g_trace.detail.clear();
    g_trace.used = 0;
    g_trace.open = false;
}

}  // namespace fnn

using namespace fnn;

#pragma GCC visibility push(default)
extern "C" {

int32_t fnn_trace_begin(int32_t max_kernels) {
    if (max_kernels < 1 || max_kernels > (1 << 20)) return FNN_E_RANGE;
    trace_release();
    g_trace.start.resize(max_kernels);
    g_trace.stop.resize(max_kernels);
    g_trace.kind.assign(max_kernels, -1);
    g_trace.detail.assign(max_kernels, 0);
    for (int i = 0; i < max_kernels; ++i) {
        if (hipEventCreate(&g_trace.start[i]) != hipSuccess || hipEventCreate(&g_trace.stop[i]) != hipSuccess) {
            g_trace.start.resize(i);
            g_trace.stop.resize(i);
            trace_release();
            return FNN_E_HIP;
        }
    }
    g_trace.open = true;
    return FNN_OK;
}

int32_t fnn_trace_end(int32_t capacity, int32_t* kinds, float* milliseconds, int32_t* details, int32_t* n_recorded) {
    if (!n_recorded || (capacity > 0 && (!kinds || !milliseconds))) return FNN_E_NULL;
    int32_t status = FNN_OK;
    const int n = g_trace.used;
    *n_recorded = n;
    for (int i = 0; i < n && i < capacity; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_trace.stop[i]) != hipSuccess ||
            hipEventElapsedTime(&ms, g_trace.start[i], g_trace.stop[i]) != hipSuccess)
            status = FNN_E_HIP;
        kinds[i] = g_trace.kind[i];
        if (details) details[i] = g_trace.detail[i];
        milliseconds[i] = ms;
    }
    trace_release();
    return status;
}

const char* fnn_trace_kind_name(int32_t kind) {
    switch (kind) {
        case TK_PREP: return "prep_kernel";
        case TK_FILL: return "fill_none_kernel";
        case TK_SEARCH: return "search_kernel";
        case TK_RECIP_STEP: return "recip_step_kernel";
        case TK_RECIP_DEDUP: return "recip_dedup_kernel";
        case TK_DENSE: return "dense_kernel";
        case TK_DENSE_FINAL: return "dense_final_kernels";
        case TK_RESOLVE: return "resolve_kernel";
        case TK_DENSE_RESOLVE: return "dense_resolve_kernels";
        case TK_BLOCKED: return "blocked_kernels";
        case TK_PIXELS: return "pairs_to_pixels_kernel";
        default: return "unknown";
    }
}

}  // extern "C"
#pragma GCC visibility pop
