/*
 * cp_probe: measurement aids (C ABI).  Not part of the method: these kernels exist so that the
 * benchmark can report, next to the published peak, the rates this very device sustains.
 *
 * cp_probe_mfma runs nothing but back-to-back v_mfma_f32_32x32x16_bf16 instructions (the
 * instruction the attention kernel is built on) on every SIMD of the device.  The matrix pipe's
 * sustained rate depends on how many operand bits toggle: the device lowers its clock under a
 * power limit, so constant operands run at the published rate and random ones do not.
 *
 * cp_probe_mix adds what the attention kernel does per MFMA besides the product: the A operand
 * is read from LDS (16 bytes per lane) and, for every second MFMA, two values go through exp2,
 * one packed conversion to bf16 and one dot2 row-sum step (per MFMA: 1 exp2, 1/2 cvt, 1/2 dot2
 * - the attention kernel's softmax per score).  No global loads, barriers or waits for fresh
 * MFMA results: it is the ceiling of that instruction mix on this device, in instruction issue
 * and in power.  In both probes the accumulators return to zero every eight trips (the B
 * operands come in pairs of opposite sign), so the values stay in a realistic range.
 */
#ifndef CP_PROBE_H
#define CP_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * operands   0: every operand element is bf16 1.0; 1: sign and mantissa from a hash of
 *            (workgroup, lane, register), magnitude in [1, 2); 2: as 1 with the exponent drawn
 *            from 2^-3 .. 2^1 as well (the spread of N(0,1) samples)
 * iters      loop trips per wavefront, a multiple of 8 in [8, 2^24]; each trip issues 8 MFMAs
 * sink       DEVICE float32 [cp_probe_mfma_sink_floats()], written (keeps the work alive)
 * stream     hipStream_t as void*, NULL = default stream
 *
 * Each call launches one kernel (256 workgroups of 8 wavefronts), asynchronously; the caller
 * times it with events on `stream`.  Algorithmic work of a launch of either kernel:
 * cp_probe_mfma_flops(iters) floating-point operations (the MFMAs only).
 * Returns 0, -1 (NULL sink), -2 (iters or operands out of range) or -4 (HIP launch error).
 */
int cp_probe_mfma(int32_t operands, int32_t iters, float *sink, void *stream);
int cp_probe_mix(int32_t operands, int32_t iters, float *sink, void *stream);
size_t cp_probe_mfma_sink_floats(void);
double cp_probe_mfma_flops(int32_t iters);

/*
 * Plain device-to-device copy of `bytes` bytes (a multiple of 16; both DEVICE pointers 16-byte
 * aligned, not overlapping), one kernel, asynchronous on `stream`: the rate HBM gives a kernel
 * that only reads and writes, to put beside the published peak.  Returns 0, -1 (NULL), -2 (size or
 * alignment) or -4 (HIP launch error).
 */
int cp_probe_copy(void *dst, const void *src, size_t bytes, void *stream);

/*
 * Test aid: fills the whole LDS (160 KiB) of every compute unit with the 32-bit `pattern`
 * (eight workgroups per compute unit, one after the other), so that the next kernel on the
 * stream starts with known leftovers.  A kernel whose result depends on LDS it did not write
 * itself shows up as a result that changes with the pattern (NaN patterns: 0x7FC07FC0,
 * 0xFFFFFFFF).  Returns 0 or -4 (HIP error).
 */
int cp_probe_fill_lds(uint32_t pattern, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CP_PROBE_H */
