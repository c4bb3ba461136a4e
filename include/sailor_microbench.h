/*
 * sailor_microbench.h -- three on-device microbenchmarks that calibrate the rooflines the plan
 * evaluator is reported against (measurement only; nothing of the method runs here).
 *
 * The evaluator's scan is bound by vector-ALU issue and its per-candidate output path by HBM
 * writes, so the ceilings are measured rather than taken from a data sheet:
 *   - a chain of dependent single-precision fused multiply-adds per lane, eight independent
 *     chains per lane (scalar-per-lane FMAs, no packed instructions): the reachable FP32 rate;
 *   - a streaming store of 16 bytes per lane over a large buffer: the reachable write bandwidth;
 *   - the same for the output format of the per-candidate evaluation: four arrays of 4, 4, 8 and
 *     4 bytes per element written side by side, one element of each per lane and step.
 *
 * All run on the current HIP device, time themselves with events on hip_stream (NULL = the
 * default stream), repeat `reps` times and report the fastest repetition.  Return 0 on
 * success, -1 for a bad argument, -2 when the buffer cannot be allocated, -3 when a HIP call
 * fails.  The write benchmarks allocate and free their buffers inside the call.
 */
#ifndef SAILOR_MICROBENCH_H
#define SAILOR_MICROBENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* workgroups of 256 lanes, each lane 8 chains of `iters` FMAs; *tflops = 2 flops per FMA */
int sailor_microbench_fma(int32_t workgroups, int32_t iters, int32_t reps, double *tflops,
                          double *best_ms, void *hip_stream);

/* `bytes` (a multiple of 4096) written once per repetition; *gbytes_per_s in 1e9 bytes/s */
int sailor_microbench_write(uint64_t bytes, int32_t reps, double *gbytes_per_s, double *best_ms,
                            void *hip_stream);

/* `elements` (at most 2^32) x 20 bytes in four arrays written once per repetition */
int sailor_microbench_write_records(uint64_t elements, int32_t reps, double *gbytes_per_s,
                                    double *best_ms, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif
