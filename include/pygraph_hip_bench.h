/*
 * pygraph_hip_bench.h -- measurement companions of libpygraph_hip (timed loops, per-kernel and
 * copy-refresh timers).  Not part of the replay path: bench.py, configs_report.py and the profiler
 * runs use them so that the loop being timed runs in C, not in the caller's interpreter.  Same
 * conventions as pygraph_hip.h.
 */
#ifndef PYGRAPH_HIP_BENCH_H
#define PYGRAPH_HIP_BENCH_H

#include "pygraph_hip.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Timed loop for benchmarks: `iters` iterations of one mode (pg_mode, 3 = pg_run_selected with
 * `mode_per_segment`, 4 = pg_replay_update), iteration t using pointer set t % n_sets of ext_sets [host]
 * ([n_sets][n_ext] device pointers), one stream synchronisation at the end; returns mean
 * microseconds per iteration measured on the host clock. */
pg_status pg_time_loop(pg_chain *chain, int32_t mode, const uint8_t *mode_per_segment,
                       const void *const *ext_sets, int32_t n_sets, int32_t iters, void *hip_stream,
                       double *us_per_iter_out);

/* The same loop with a HIP event after every iteration: us_each_out [host] receives `iters`
 * completion-to-completion times in microseconds (for medians and spreads; the events add a marker
 * per iteration to the stream, so their mean is slightly above pg_time_loop's). */
pg_status pg_time_loop_each(pg_chain *chain, int32_t mode, const uint8_t *mode_per_segment,
                            const void *const *ext_sets, int32_t n_sets, int32_t iters, void *hip_stream,
                            float *us_each_out);

/* GPU execution time of each kernel: launches kernels [k_begin, k_end) eagerly (as pg_eager_range
 * does), each with a pair of events that take the kernel's own start and end timestamps,
 * synchronises the stream, and writes k_end - k_begin durations in microseconds to dur_us_out
 * [host].  For roofline figures: time between launches is not included. */
pg_status pg_time_kernels(pg_chain *chain, const void *const *ext_dev_ptrs, int32_t k_begin, int32_t k_end,
                          void *hip_stream, float *dur_us_out);

/* GPU execution time of one copy refresh (the batched copy kernel's launches, summed), measured the
 * same way; *dur_us_out [host] in microseconds.  Synchronises the stream. */
pg_status pg_time_refresh_copy(pg_chain *chain, const void *const *ext_dev_ptrs, void *hip_stream, float *dur_us_out);

#ifdef __cplusplus
}
#endif
#endif
