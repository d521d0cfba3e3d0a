/*
 * spes_bench.h -- benchmark aids exported by the SPES library next to the entry points of spes.h.
 *
 * These calls exist for bench.py: a matrix-rate reference loop and per-stage timing of the layer's
 * forward and backward.  Unlike everything in spes.h the stage timing keeps process-wide state (a
 * set of HIP events); it holds no device memory.  Not meant for production paths.
 */
#ifndef SPES_BENCH_H_
#define SPES_BENCH_H_

#include "spes.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Reference rate of the matrix cores, for benchmarks: launches `blocks` workgroups of four
 * wavefronts that each run `iters` rounds of sixty-four 16x16x32 bf16 MFMAs on operands held in
 * registers, taken from `data`.  The shader clock under matrix load depends on the operand
 * values (power), so the rate to compare a GEMM with is this loop timed on values like the
 * GEMM's.  The caller times the launch (events on `stream`); *flop receives the number of
 * floating-point operations it performs.
 *
 *  data   DEVICE, 64 KiB of bf16 operand values     sink  DEVICE [blocks] f32 out (no meaning)
 *  flop   HOST out, may be NULL
 */
SPES_API int spes_ref_mfma_rate(const void* data, int32_t blocks, int32_t iters, float* sink,
                                double* flop, void* stream);

/* Stage timing for benchmarks.  While enabled, spes_moe_fwd / spes_moe_bwd record a
 * HIP event on the caller's stream after each of their stages (the steps of the hot
 * path: router GEMM, softmax/top-k, histogram/scan/rank, the grouped GEMMs,
 * combine, ...).  spes_profile_read waits for the last recorded event of the most
 * recent forward (which=0) or backward (which=1) and returns the number of stages,
 * filling ms[i] (milliseconds) and names[i] (static strings; names may be NULL) for
 * at most cap stages.  The events are the library's only process-wide state; calls
 * that overlap on several streams while timing is enabled overwrite each other's
 * records.  Not meant for production paths. */
SPES_API int spes_profile_enable(int32_t on);
SPES_API int spes_profile_read(int32_t which, float* ms, const char** names, int32_t cap);

#ifdef __cplusplus
}
#endif
#endif /* SPES_BENCH_H_ */
