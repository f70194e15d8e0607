/*
 * fnn_measure.h -- measurement aids of libfnn.  Nothing here is part of the matching path
 * (include/fnn.h): these calls exist for the benchmark and the tests, hold process-wide state
 * and may wait for the device.
 */
#ifndef FNN_MEASURE_H
#define FNN_MEASURE_H

#include "fnn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Per-kernel timing.  Between
 * fnn_trace_begin and fnn_trace_end every kernel the library launches -- up to max_kernels,
 * later ones run untimed -- carries its own pair of HIP events, so that fnn_trace_end can
 * report each kernel's device-side duration.  fnn_trace_end waits for the traced kernels,
 * writes min(*n_recorded, capacity) entries (kinds[i] names the kernel, see
 * fnn_trace_kind_name; milliseconds[i] is its duration, in launch order; details[i], if the
 * array is not NULL, is the launch shape the host chose: for a search the number of groups of
 * four 32-query blocks a wave keeps resident, plus 100 when the kernel that stages the candidate
 * tiles through LDS ran; for the dense pass-1 kernel 1 when the variant that stages the query
 * blocks through LDS ran; 0 otherwise) to HOST
 * arrays and closes the trace.  The trace is process-wide state and not thread-safe, and must
 * not be open during HIP graph capture.
 */
int32_t fnn_trace_begin(int32_t max_kernels);
int32_t fnn_trace_end(int32_t capacity, int32_t* kinds, float* milliseconds, int32_t* details, int32_t* n_recorded);
const char* fnn_trace_kind_name(int32_t kind);

/*
 * The time this device
 * needs per 32x32 block of scores for the bare instruction mix of the kernels, in a loop that
 * touches registers only -- the yardstick the kernels' own times are held against.
 *   mix 0: one K=16 fp16 matrix instruction per block (16 channels)
 *   mix 1: a K=16 and a K=8 instruction (the 24-channel block of the paper's d = 24)
 *   mix 2: two K=16 instructions (a 32-channel block)
 *   mix 3: mix 1 plus the eight 3-input maxima that fold a block (search kernel arithmetic)
 *   mix 4: mix 1 plus sixteen 3-input maxima per block (dense kernel arithmetic)
 *   mix 5: the block as four 16x16x32 fp16 instructions (24 channels padded to 32)
 *   mix 6, 7, 8: mixes 1, 3, 4 on the bfloat16 instructions
 * Runs two waves on every SIMD of the current device, each doing blocks_per_wave blocks
 * (>= 4), three times, WAITS for them, and writes the best time as nanoseconds per block and
 * SIMD to *ns_per_block (host).  scratch: device memory, 4-byte aligned, at least
 * 2048 bytes per compute unit (one word per thread is stored there).
 * Errors: FNN_E_NULL, FNN_E_RANGE (mix, blocks_per_wave), FNN_E_WORKSPACE, FNN_E_HIP.
 */
int32_t fnn_measure_ceiling(int32_t mix, int32_t blocks_per_wave, void* scratch, size_t scratch_bytes,
                            float* ns_per_block, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FNN_MEASURE_H */
