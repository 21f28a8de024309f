/*
 * dmath_measure.h -- measurement aids of the dMath GEMM / convolution library.  Nothing here is
 * part of the paper's method or of the product interface (dmath.h); bench and profiling programs
 * use these calls to put the kernels' timings beside what the matrix cores sustain and to read a
 * kernel's own cycle counts.  Same conventions as dmath.h: a status is returned, nothing throws,
 * out-parameters are untouched on error.
 */
#ifndef DMATH_MEASURE_H
#define DMATH_MEASURE_H

#include "dmath.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement aid, for builds of the library made with -DDMATH_CYCLE_PROBE only (the product
 * library returns DMATH_ERR_UNSUPPORTED): after a specialised fp16 dmath_gemm, waits for
 * the stream and returns what wavefront 0 of the workgroup owning C tile (0,0) (first k-split) counted:
 * out6[0..2] shader-clock cycles of prologue, k-loop, epilogue; out6[3] cycles waiting at the
 * per-k-tile barrier; out6[4] elapsed ticks of the 100 MHz reference clock; out6[5] k-tiles.
 * (cycles / ticks * 100 MHz = the clock the kernel ran at.)
 */
dmath_status_t dmath_cycle_probe_read(dmath_ctx_t ctx, uint64_t *out6);

/*
 * Measurement aid (not part of the paper's method): enqueues a register-only kernel in which
 * every wavefront issues independent chains of the MFMA instruction the GEMM kernels of
 * `dtype` use (fp16: v_mfma_f32_16x16x32_f16, 64 per iteration; fp32 and fp64: 16 per iteration),
 * `iters` iterations per wavefront, and returns in *flops the number
 * of floating-point operations it performs.  Timing it gives the matrix-core rate the chip
 * sustains at its clocks under load, to be read beside the nominal peak.
 */
dmath_status_t dmath_mfma_peak_probe(dmath_ctx_t ctx, dmath_dtype_t dtype, int32_t iters,
                                     double *flops);

/*
 * The same for fp16 on v_mfma_f32_32x32x16_f16 (16 per iteration, the same flops per iteration):
 * the instruction of the fp16 convolution kernels and of the 64-row GEMM tiles.  Read beside
 * dmath_mfma_peak_probe(DMATH_F16) it shows what the smaller instruction buys at the chip's
 * power limit.
 */
dmath_status_t dmath_mfma_peak_probe_f16_32x32x16(dmath_ctx_t ctx, int32_t iters, double *flops);

#ifdef __cplusplus
}
#endif
#endif /* DMATH_MEASURE_H */
