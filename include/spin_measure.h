/*
 * spin_measure.h -- measurement aids of libspin.so.  Nothing here is part of the method: these
 * calls exist so that a benchmark can time the library's kernels one by one and compare them with
 * what a plain read reaches on the same machine.  The method's calls are in spin.h.
 */
#ifndef SPIN_MEASURE_H
#define SPIN_MEASURE_H

#include "spin.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing for benchmarks.  spin_profile_enable(ctx, capacity > 0)
 * creates `capacity` HIP event pairs per kernel; from then on each kernel
 * launch of a stage call carries a start and a stop event on its stream (up to
 * `capacity` launches per kernel, later ones are not timed).
 * spin_profile_read() waits for the recorded events of kernel `which`, returns
 * how many launches were timed and their mean and minimum duration in
 * microseconds, and resets that kernel's counter.  capacity == 0 disables and
 * releases the events.  Not for concurrent use with stage calls. */
enum spin_kernel_id {
  SPIN_K_SCORE = 0, SPIN_K_SELECT = 1, SPIN_K_RESOLVE = 2, SPIN_K_DECODE = 3, SPIN_K_MERGE = 4,
  SPIN_K_INDEX = 5, SPIN_K_PACK = 6, SPIN_K_GATHER = 7, SPIN_K_PROBE = 8,
  SPIN_K_SELECT_HIST = 9, /* first launch of stage 2 for rows of more than 16384 partitions */
  SPIN_K_OFFLOAD = 10, SPIN_K_APPEND = 11,
  SPIN_K_META = 12 /* spin_reclaim_tail, spin_alloc_leaves, spin_free_leaves */
};
int spin_profile_enable(spin_ctx *ctx, int32_t capacity);
int spin_profile_read(spin_ctx *ctx, int32_t which, int32_t *count, float *mean_us, float *min_us);

/* Measurement aid: streams `bytes` (a multiple of 16) from the DEVICE buffer `buf`
 * with a plain read-only kernel, timed as SPIN_K_PROBE when profiling is enabled.
 * Gives the bandwidth a single launch of that size can reach on the box at hand,
 * the yardstick the stage kernels are compared with. */
int spin_probe_stream_read(spin_ctx *ctx, const void *buf, size_t bytes, void *workspace, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPIN_MEASURE_H */
