/*
 * ifkv_calibrate.h -- calibration kernels of libifkv (not part of the method).
 *
 * The benchmark times these on the machine it runs on, to state what the
 * hardware delivers next to the published peaks, and scales hardware-counter
 * readings by what the same counters read for the plain copy.
 */
#ifndef IFKV_CALIBRATE_H
#define IFKV_CALIBRATE_H

#include "ifkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Calibration utility (not part of the method): a plain streaming copy of
 * n_bytes (multiple of 16, both pointers 16-byte aligned, device memory) with
 * the same load/store shape the streaming stages use.  The benchmark times it
 * to state the HBM bandwidth the machine actually delivers next to the
 * published peak, and hardware-counter readings are scaled by what the same
 * counters read for this kernel.
 */
int ifkv_copy_bytes(ifkv_ctx *ctx, void *dst, const void *src, int64_t n_bytes);

/*
 * Calibration utility (not part of the method): a loop of independent
 * 32x32x16 bf16 MFMAs on register-resident operands, two wavefronts per SIMD on
 * every compute unit.  The benchmark times it to state what the matrix pipes
 * sustain on this machine next to the published peak.
 *   pattern     0: every operand element is 1.0 (least switching activity);
 *               1: pseudo-random sign and mantissa, magnitudes in [0.5, 2)
 *   iterations  loop trips per wavefront, 1 .. 10^7 (32 MFMAs per trip)
 *   sink        device, at least ifkv_mfma_probe_sink_floats() floats; receives
 *               one checksum per thread (content is not meaningful)
 *   flops_out   host, nullable: floating-point operations one launch performs
 * Errors: IFKV_EINVAL for a NULL ctx or sink, an unknown pattern or an
 * iteration count out of range.
 */
int ifkv_mfma_probe(ifkv_ctx *ctx, int pattern, int64_t iterations, float *sink, double *flops_out);
int64_t ifkv_mfma_probe_sink_floats(void);

#ifdef __cplusplus
}
#endif
#endif /* IFKV_CALIBRATE_H */
