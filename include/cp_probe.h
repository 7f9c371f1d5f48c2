/*
 * cp_probe: measurement aids (C ABI).  Not part of the method: these kernels exist so that the
 * benchmark can report, next to the published peak, the rate this very device sustains.
 *
 * cp_probe_mfma runs nothing but back-to-back v_mfma_f32_32x32x16_bf16 instructions (the
 * instruction the attention kernel is built on) on every SIMD of the device, either on
 * constant operands or on operands whose sign and mantissa bits look random.  The matrix
 * pipe's sustained rate depends on how many operand bits toggle (power), so the second figure
 * is the realistic ceiling for a bf16 kernel working on real data.
 */
#ifndef CP_PROBE_H
#define CP_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * random_operands  0: every operand element is bf16 1.0; 1: sign and mantissa from a hash of
 *                  (workgroup, lane, register), magnitude in [1, 2)
 * iters            loop trips per wavefront, 1 <= iters <= 2^24; each trip issues 8 MFMAs
 * sink             DEVICE float32 [cp_probe_mfma_sink_floats()], written (keeps the work alive)
 * stream           hipStream_t as void*, NULL = default stream
 *
 * Launches one kernel, asynchronously; the caller times it with events on `stream`.
 * Algorithmic work of the launch: cp_probe_mfma_flops(iters) floating-point operations.
 * Returns 0, -1 (NULL sink), -2 (iters out of range) or -4 (HIP launch error).
 */
int cp_probe_mfma(int32_t random_operands, int32_t iters, float *sink, void *stream);
size_t cp_probe_mfma_sink_floats(void);
double cp_probe_mfma_flops(int32_t iters);

#ifdef __cplusplus
}
#endif
#endif /* CP_PROBE_H */
