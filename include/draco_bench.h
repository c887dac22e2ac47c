/*
 * draco_bench.h -- measuring instruments of the DRACO library: a calibration
 * copy kernel and per-kernel timing.  None of this is part of the method's
 * boundary (include/draco.h); the benchmark and the profiles use it.
 */
#ifndef DRACO_BENCH_H
#define DRACO_BENCH_H

#include "draco.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Plain device-to-device copy of a [rows][ld] fp32 slab (row_len floats used
 * per row; row_len and ld multiples of 4, pointers 16-byte aligned; rows <=
 * 65535) with 16-byte non-temporal accesses, one 4 KiB piece of one row per
 * workgroup, pieces of a row varying fastest: a calibration kernel, the fastest
 * slab copy found on this GPU.  Timing it gives the copy bandwidth the GPU
 * sustains (the ceiling of the encoders, which read and write equal amounts);
 * profiling it gives the scale of the hardware byte counters for a known
 * 2*4*rows*row_len bytes.  Asynchronous on `stream`. */
int draco_copy_probe(const float* src_dev, float* dst_dev, int rows, int64_t row_len, int64_t ld,
                     void* stream);

/* Kernel timing with HIP events recorded on the stream each kernel is launched
 * on.  draco_plan_set_timing(plan, n) gives every kernel kind n event pairs
 * (n = 0 switches timing off); from then on each launch of a kind uses the next
 * free pair (launches beyond n are not timed) and nothing waits.
 * draco_plan_kernel_time waits for the recorded kernels of one kind, returns
 * their summed duration in milliseconds and their number, and frees the pairs
 * for reuse.  draco_plan_kernel_times does the same but writes each launch's
 * duration, in launch order, to ms_host[0 .. min(*launches, capacity)).
 * kind: 0 encode, 1 repetition vote, 2 cyclic projection (with its small
 * reduction), 3 cyclic recombination, 4 the cyclic locator (phi steps 2-4 and
 * b, one wavefront). */
int draco_plan_set_timing(draco_plan* plan, int max_records);
int draco_plan_kernel_time(draco_plan* plan, int kind, double* total_ms, int* launches);
int draco_plan_kernel_times(draco_plan* plan, int kind, double* ms_host, int capacity,
                            int* launches);

#ifdef __cplusplus
}
#endif
#endif /* DRACO_BENCH_H */
