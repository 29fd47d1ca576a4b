/* hexa_moe_bench.h -- measurement helpers of libhexa_moe.  NOT part of the layer's interface
 * (include/hexa_moe.h): bench.py uses them to time the library's kernels one by one and to
 * measure the matrix rate the part sustains.  They live in the same shared library because they
 * have to bracket the library's own launches. */
#ifndef HEXA_MOE_BENCH_H
#define HEXA_MOE_BENCH_H

#include "hexa_moe.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing.  While enabled, every kernel the library launches is bracketed by two HIP
 * events on its stream; enabling (or disabling) discards earlier records.  This is the only part
 * of the library that creates HIP objects, so it must stay off under stream capture.
 * hexa_moe_profile_read(i, ...) waits for the recorded events and returns the i-th distinct
 * kernel label with its summed duration in ms and its launch count; returns 0 once i is past
 * the last label (or on a HIP error), else 1.  The record list is guarded by a mutex; the
 * recording state is process-wide. */
HEXA_API void hexa_moe_profile_enable(int on);
HEXA_API int hexa_moe_profile_read(int i, const char **label, float *ms_total, int *launches);

/* Enqueues a register-only bf16 MFMA loop: `workgroups` workgroups of four wavefronts, each wavefront
 * issuing iters * 32 16x16x32 MFMAs (variant 2: iters * 16 32x32x16 MFMAs; the same FLOP), and writes
 * the FLOP count of the launch to *flop (host).  Timed by the caller on `stream`, it gives the matrix
 * rate the part sustains under its power limit, which depends on the operand bits:
 *   variant 0  16x16x32, pseudo-random operands of the layer's magnitude (what bench.py reports)
 *   variant 1  16x16x32, all-zero operands
 *   variant 2  32x32x16, pseudo-random operands
 * sink: dev, >= 4 bytes, never written in practice. */
HEXA_API hexa_status hexa_moe_mfma_probe(int32_t variant, int32_t workgroups, int32_t iters, float *sink,
                                void *stream, double *flop);

#ifdef __cplusplus
}
#endif
#endif /* HEXA_MOE_BENCH_H */
