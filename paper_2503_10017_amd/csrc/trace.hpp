// Optional per-kernel timing: when a trace is open every kernel launch of the library is
// bracketed by a pair of HIP events attached to the dispatch itself, so the elapsed time of
// a pair is that kernel's own duration.  Closed (the default), launches are plain.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

namespace fnn {

enum TraceKind : int {
    TK_PREP = 0,
    TK_FILL = 1,
    TK_SEARCH = 2,
    TK_RESERVED_3 = 3,  // numbers are part of what fnn_trace_end reports: retired kinds keep theirs
    TK_RESERVED_4 = 4,
    TK_RECIP_STEP = 5,
    TK_RECIP_DEDUP = 6,
    TK_DENSE = 7,
    TK_DENSE_FINAL = 8,
    TK_RESOLVE = 9,
    TK_DENSE_RESOLVE = 10,
    TK_BLOCKED = 11,
    TK_PIXELS = 12,
    TK_COUNT = 13
};

// Returns false when no trace is open or it is full; otherwise hands out the next event pair.
// `detail` is a number the launcher wants reported with the kernel (the launch shape it chose).
bool trace_next(int kind, int detail, hipEvent_t* start, hipEvent_t* stop);

template <typename Kernel, typename... Args>
inline hipError_t launch_detail(int kind, int detail, Kernel kernel, dim3 grid, dim3 block, size_t lds_bytes,
                                hipStream_t s, Args... args) {
    hipEvent_t e0, e1;
    if (trace_next(kind, detail, &e0, &e1)) {
        hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, s, e0, e1, 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, s, args...);
    }
    return hipGetLastError();
}
template <typename Kernel, typename... Args>
inline hipError_t launch(int kind, Kernel kernel, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t s, Args... args) {
    return launch_detail(kind, 0, kernel, grid, block, lds_bytes, s, args...);
}

}  // namespace fnn
