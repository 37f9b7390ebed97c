/*
 * libitq3s -- measurement aids.  NOT part of the product interface (include/itq3s.h): these calls
 * exist for the benchmark and the profiles.  Unlike everything in itq3s.h they create and destroy
 * HIP events and WAIT for the device, so they are not for production loops and cannot be captured
 * in a graph.  They cite no passage of the paper: they compute nothing of their own.
 */
#ifndef ITQ3S_BENCH_H
#define ITQ3S_BENCH_H

#include "itq3s.h"

#ifdef __cplusplus
extern "C" {
#endif

/* itq3s_matmul / itq3s_matmul_grouped with the same arguments, after which the call WAITS for the
 * work and stores in *kernel_ms (HOST pointer, required) the duration of the contraction kernel
 * alone (the streaming kernel for M <= 16, its first pass for M <= 32; for larger M the first tiled
 * launch; not the activation-rotation launch in front of it, not the launch that adds up partial
 * sums behind it for shapes with few tiles, not launch gaps), taken from HIP events attached to that
 * kernel's dispatch. */
int itq3s_matmul_timed(const uint32_t *codes, const uint32_t *scales, int64_t N, int64_t K, const void *X, int64_t M,
                       int64_t ldx, void *Y, int y_dtype, int64_t ldy, void *workspace, size_t workspace_bytes,
                       uint32_t *status_flags, void *stream, float *kernel_ms);

int itq3s_matmul_grouped_timed(const itq3s_weight *w, int count, int64_t K, const void *X, int64_t M, int64_t ldx,
                               int y_dtype, void *workspace, size_t workspace_bytes, uint32_t *status_flags,
                               void *stream, float *kernel_ms);

/* itq3s_matmul_weight_side, then wait; *kernel_ms (HOST pointer, required) = the kernel's duration. */
int itq3s_matmul_weight_side_timed(const uint32_t *codes, const uint32_t *scales, int64_t N, int64_t K, const void *X,
                                   int64_t M, int64_t ldx, void *Y, int y_dtype, int64_t ldy, uint32_t *status_flags,
                                   void *stream, float *kernel_ms);

/* A plain streaming read of `bytes` bytes (rounded down to a multiple of 16) of device memory at src
 * (16-byte aligned), nothing else -- the time such a launch takes is the practical floor for a
 * streaming matmul over the same bytes.  sink: one device uint32 (written only for one particular
 * checksum of the data; present so that the reads cannot be optimised away).  Does not wait. */
int itq3s_read_probe(const void *src, size_t bytes, uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ITQ3S_BENCH_H */
