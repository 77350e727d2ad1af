/*
 * wq_measure.h -- measurement aids of libwq (not part of the WindowQuant method).
 *
 * What a benchmark needs beside the calls of wq.h: the decode kernel timed on its own, the achievable HBM read rate
 * of the GPU (also the reference that hardware byte counters are scaled by) and the matrix-core rate on register
 * operands.  Same conventions as wq.h (device pointers, host scalars, work enqueued on the context's stream).
 */
#ifndef WQ_MEASURE_H
#define WQ_MEASURE_H

#include "wq.h"

#ifdef __cplusplus
extern "C" {
#endif

/* or-ed into algo: run only the kernel that streams the cache and leave its per-split partials in the workspace
 * (out and lse are not written).  A measurement aid: it lets that kernel be timed without the merge kernel.   */
#define WQ_DECODE_PARTIALS_ONLY 0x100
/* ---- timing of the dominant kernel (measurement aid) ---------------------------------------------------------
 * With timing enabled every wq_decode_attention records a HIP event right before and right after its main
 * kernel (the one that streams the cache) on the context's stream, in a ring of 64 event pairs created once by
 * wq_decode_timing(ctx, 1); the decode call itself still allocates nothing and does not synchronise.
 * wq_decode_times_us waits for the last timed call and returns the durations of the last n (<= 64) timed calls,
 * oldest first, in microseconds.  Enabling or disabling restarts the count.                                   */
int wq_decode_timing(wq_ctx* ctx, int enable);
int wq_decode_times_us(wq_ctx* ctx, float* us, int n);

/* ---- measurement probes (not part of the method; for callers that cannot time a plain kernel themselves) ----
 * wq_probe_stream streams `bytes` (multiple of 16) of device memory with 16-byte loads from `blocks` workgroups of 256 lanes:
 * read-only when dst is NULL, a plain copy otherwise.  Gives the achievable HBM rate and the reference that
 * hardware byte counters are scaled by.                                                                       */
int wq_probe_stream(wq_ctx* ctx, const void* src, void* dst, int64_t bytes, int blocks);
/* Runs `workgroups` x 8 wavefronts of `iters` (a multiple of 4) x 32 independent v_mfma_f32_16x16x32_bf16 products on register
 * operands (no memory traffic): all ones when random_operands == 0, else random values that change from product to
 * product.  Gives the matrix-core rate this GPU sustains, which depends on the data (the clock drops under
 * load): the figure the pairwise scoring kernel is to be read against.  *flops (host, may be NULL) receives the
 * floating-point operations of the launch.  Needs a workspace (one word of it is the kernel's sink).               */
int wq_probe_mfma(wq_ctx* ctx, int random_operands, int workgroups, int iters, double* flops);

#ifdef __cplusplus
}
#endif
#endif /* WQ_MEASURE_H */
