/*
 * specasr_profile.h -- measurement aids of the tree-verification library.
 *
 * Not part of the verification path (include/specasr.h): these calls let a benchmark time one
 * projection GEMM per forward with HIP events attached to that dispatch on the caller's stream.
 * They have no effect on results.
 */
#ifndef SPECASR_PROFILE_H
#define SPECASR_PROFILE_H

#include "specasr.h"

#ifdef __cplusplus
extern "C" {
#endif

/* While enabled, every forward
 * launches ONE instance of the chosen projection GEMM (the layer rotates from call to call)
 * with a pair of HIP events that take the start and stop time of that dispatch on the caller's
 * stream (enable = 2: only the launches of the tiled kernel that prefill passes over more than 64
 * rows use).  specasr_stage_time waits for the recorded events and returns the accumulated
 * kernel milliseconds and the number of launches measured since profiling was enabled, plus the
 * weight bytes one such launch streams; specasr_stage_rows returns the activation rows summed
 * over the same launches (their algorithmic flops are 2 x rows x weight elements). */
typedef enum { SPECASR_STAGE_QKV = 0, SPECASR_STAGE_O = 1, SPECASR_STAGE_GATE_UP = 2,
               SPECASR_STAGE_DOWN = 3, SPECASR_STAGE_LM_HEAD = 4 } specasr_stage;
specasr_status specasr_profile_stage(specasr_ctx *ctx, int32_t stage, int32_t enable);
specasr_status specasr_stage_time(specasr_ctx *ctx, double *total_ms, int64_t *launches,
                                  double *weight_bytes_per_launch);
specasr_status specasr_stage_rows(specasr_ctx *ctx, int64_t *rows);

/* Measured read ceiling: streams `bytes` (>= 1 MiB, 16-byte aligned DEVICE buffer, read only -- it
 * should be far larger than the 256 MB Infinity Cache) `reps` times on `stream` with the weight
 * stream's access pattern and no arithmetic, synchronises, and returns GB/s -- what a benchmark
 * quotes next to the nominal HBM bandwidth. */
specasr_status specasr_read_ceiling(specasr_ctx *ctx, const void *buf_dev, size_t bytes, int32_t reps,
                                    void *stream, double *gb_per_s);

#ifdef __cplusplus
}
#endif
#endif /* SPECASR_PROFILE_H */
