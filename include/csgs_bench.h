/*
 * csgs_bench -- measuring aids of the csgs library (see csgs.h for the method's own entry points).
 * None of these is part of the sampled layer step: per-kernel timing of the library's launches, and
 * three yardstick kernels (streaming copy, scattered 64-bit atomic adds, back-to-back matrix
 * instructions) against which a benchmark states what the step's kernels reach.
 * Conventions as in csgs.h: device pointers unless marked host, work enqueued on `stream`,
 * CSGS_OK or a negative CSGS_E* code.
 */
#ifndef CSGS_BENCH_H
#define CSGS_BENCH_H

#include "csgs.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Per-kernel timing for benchmarks (off by default).  While enabled, every kernel launch of the
 * library carries two HIP events that the runtime stamps with the start and the end of that
 * dispatch.  csgs_profile_collect, called after the caller has synchronised, fills ms_sum[k] /
 * launches[k] (host arrays of csgs_profile_kernel_count() entries) with the summed kernel
 * durations in milliseconds and the number of launches per kernel since the last collect, and
 * resets.  Process-wide, not thread-safe; creates HIP events on first use, so it is not for
 * callers that may not allocate.
 */
int csgs_profile_enable(int on);
int csgs_profile_kernel_count(void);
const char *csgs_profile_kernel_name(int kernel);
int csgs_profile_collect(double *ms_sum /*host*/, int64_t *launches /*host*/);
/* The same launch by launch, for medians and percentiles: fills ms[i] / kernel[i] (host arrays of
 * `cap` entries) with the duration and the kernel index of the first min(cap, n) launches since the
 * last collect, stores n (all launches timed since then) in *n_out, and does NOT reset -- call it
 * before csgs_profile_collect. */
int csgs_profile_samples(float *ms /*host*/, int32_t *kernel /*host*/, int64_t cap, int64_t *n_out /*host*/);

/* Plain device-to-device copy of `bytes` bytes (a multiple of 16, both pointers 16-byte aligned)
 * with an ordinary streaming kernel: the yardstick for achievable HBM bandwidth, and the
 * known-size kernel against which hardware byte counters are calibrated. */
int csgs_calib_copy(void *dst, const void *src, size_t bytes, void *stream);

/* n_updates fire-and-forget 64-bit integer atomic adds (+1, device scope) to pseudo-random entries of
 * `table` (n_table entries, device, 8-byte aligned, contents are modified): the yardstick for the
 * weight scan of csgs_build_probs, which updates its per-node accumulators the same way. */
int csgs_calib_atomics(uint64_t *table, size_t n_table, size_t n_updates, void *stream);

/* n_reads independent 8-byte reads of pseudo-random entries of `table` (n_table entries, device, 8-byte aligned): what a
 * random lookup costs in time and in fetched bytes.  csgs_sample_layer looks up one such entry per scanned edge (the node ->
 * position table).  `sink` (device, n_sink >= 4 194 304 entries) receives one value per thread so that the reads are kept. */
int csgs_calib_lookups(const uint64_t *table, size_t n_table, size_t n_reads, uint64_t *sink, size_t n_sink, void *stream);

/* Matrix-core yardstick for csgs_layer_gemm: CSGS_CALIB_MFMA_BLOCKS blocks of four wavefronts, each
 * wavefront issuing 64 * iters double-precision 16 x 16 x 4 matrix instructions (2048 flops each) on
 * eight independent accumulators, i.e. CSGS_CALIB_MFMA_BLOCKS * 4 * 64 * 2048 * iters flops per call.
 * from_lds = 0: operands stay in registers (what the matrix cores sustain); from_lds = 1: every 64
 * instructions the operands are re-read from LDS as floats and widened, which is the inner loop of
 * the layer GEMM without its global loads and barriers.  `sink` (device, n_sink >=
 * CSGS_CALIB_MFMA_BLOCKS * 256 doubles) receives one value per thread so that the work is kept. */
#define CSGS_CALIB_MFMA_BLOCKS 2048
int csgs_calib_mfma_f64(double *sink, size_t n_sink, int64_t iters, int32_t from_lds, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CSGS_BENCH_H */
