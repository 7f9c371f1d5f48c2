// cp_probe: measurement aids behind the C ABI of cp_probe.h.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <mutex>

#include "cp_probe.h"

namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kBlocks = 256;  // one workgroup of eight wavefronts per compute unit, as the attention kernel
constexpr int kThreads = 512;
constexpr int kMfmaPerTrip = 8;
constexpr int kLdsVectors = 8192; // 128 KiB of operand data in LDS for the mix probe

__device__ inline unsigned mix(unsigned x)
{
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}
// Two bf16 values: kind 0 -> 1.0; kind 1 -> random sign and mantissa, exponent of 1.0; kind 2 ->
// random sign and mantissa and an exponent drawn from 2^-3 .. 2^1 (the spread of N(0,1) samples)
__device__ inline unsigned operand_pair(int kind, unsigned seed)
{
    if (kind == 0) return 0x3f803f80u;
    const unsigned r = mix(seed) & 0x807f807fu;
    if (kind == 1) return r | 0x3f803f80u;
    const unsigned e0 = 124u + mix(seed * 3u + 1u) % 5u, e1 = 124u + mix(seed * 3u + 2u) % 5u;
    return r | (e0 << 7) | (e1 << 23);
}

// Eight independent accumulator tiles per wavefront, so that consecutive MFMAs never wait for
// each other; the B operand rotates so that the loop cannot be folded.  The trip loop is
// unrolled eight times so that every register index is a constant.
//
// kMix adds, per MFMA, what the attention kernel does per MFMA besides the product itself: the A
// operand comes from LDS (one 16-byte read per lane) and, for every second MFMA, two scores go
// through exp2, one packed conversion to bf16 and one dot2 row-sum step.  There are no global
// loads, barriers or dependencies on fresh MFMA results: it is the rate of that instruction mix
// when nothing else is in its way.  The B operands come in pairs of opposite sign, so that the
// accumulators return to zero every eight trips and the "scores" stay in a realistic range.
template <bool kMix>
__global__ __launch_bounds__(kThreads) void mfma_stream_kernel(float *sink, int iters, int kind)
{
    __shared__ __attribute__((aligned(16))) u32x4 lds[kMix ? kLdsVectors : 1];
    f32x16 acc[kMfmaPerTrip];
    u32x4 a[kMfmaPerTrip], b[kMfmaPerTrip];
    if (kMix) {
        for (int i = threadIdx.x; i < kLdsVectors; i += kThreads) {
            u32x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = operand_pair(kind, (unsigned)i * 4u + e + blockIdx.x * 77777u);
            lds[i] = v;
        }
    }
#pragma unroll
    for (int i = 0; i < kMfmaPerTrip; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const unsigned seed = (blockIdx.x * kThreads + threadIdx.x) * 64u + (i & 3) * 8u + e;
            a[i][e] = operand_pair(kind, seed + i * 1000u);
            b[i][e] = operand_pair(kind, seed + 4u);
            if (kind != 0 && i >= 4) b[i][e] ^= 0x80008000u; // b[i + 4] = -b[i]
        }
    }
    __syncthreads();
    float psum = 0.f;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    const int lane_off = (threadIdx.x & 63) + (threadIdx.x >> 6) * 1024;
    for (int it = 0; it < iters; it += 8) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
#pragma unroll
            for (int i = 0; i < kMfmaPerTrip; ++i) {
                u32x4 av = a[i];
                if (kMix) av = lds[lane_off + ((i + u * 8) & 15) * 64];
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av),
                                                                 __builtin_bit_cast(bf16x8, b[(i + u) & 7]), acc[i],
                                                                 0, 0, 0);
                if (kMix && (i & 1)) {
                    f32x2 x; // "scores": elements of an accumulator that was written four MFMAs ago
                    x[0] = __builtin_amdgcn_exp2f(acc[(i + 4) & 7][u]);
                    x[1] = __builtin_amdgcn_exp2f(acc[(i + 4) & 7][u + 8]);
                    const bf16x2 y = __builtin_convertvector(x, bf16x2);
                    psum = __builtin_amdgcn_fdot2_f32_bf16(y, ones, psum, false);
                }
            }
        }
    }
    float r = psum;
#pragma unroll
    for (int i = 0; i < kMfmaPerTrip; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) r += acc[i][v];
    sink[blockIdx.x * kThreads + threadIdx.x] = r;
}

// Plain device copy: every thread moves four 16-byte pieces per step (four loads in flight before
// the first store), streaming hints on both sides: what HBM gives a kernel that does nothing else.
constexpr int kCopyUnroll = 4;
__global__ __launch_bounds__(256) void copy_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src, size_t n)
{
    const size_t stride = (size_t)gridDim.x * 256 * kCopyUnroll;
    for (size_t base = (size_t)blockIdx.x * 256 * kCopyUnroll + threadIdx.x; base < n; base += stride) {
        u32x4 v[kCopyUnroll];
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u)
            if (base + u * 256 < n) v[u] = __builtin_nontemporal_load(src + base + u * 256);
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u)
            if (base + u * 256 < n) __builtin_nontemporal_store(v[u], dst + base + u * 256);
    }
}

// Every thread writes its share of the 160 KiB and reads it back (so that the stores cannot be
// dropped); the flag is never set for a pattern the caller can pass twice in one word.
constexpr int kLdsFillBytes = 160 * 1024;
__global__ __launch_bounds__(1024) void fill_lds_kernel(unsigned pattern, unsigned *flag)
{
    extern __shared__ unsigned fill_words[];
    for (int i = threadIdx.x; i < kLdsFillBytes / 4; i += 1024) fill_words[i] = pattern;
    __syncthreads();
    unsigned x = 0;
    for (int i = threadIdx.x; i < kLdsFillBytes / 4; i += 1024) x |= fill_words[i] ^ pattern;
    if (x != 0 && flag) *flag = x;
}

int launch(bool with_mix, int32_t operands, int32_t iters, float *sink, void *stream)
{
    if (!sink) return -1;
    if (iters < 8 || iters > (1 << 24) || iters % 8 != 0 || operands < 0 || operands > 2) return -2;
    hipStream_t hs = (hipStream_t)stream;
    if (with_mix) hipLaunchKernelGGL(mfma_stream_kernel<true>, dim3(kBlocks), dim3(kThreads), 0, hs, sink, iters, operands);
    else hipLaunchKernelGGL(mfma_stream_kernel<false>, dim3(kBlocks), dim3(kThreads), 0, hs, sink, iters, operands);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

} // namespace

extern "C" size_t cp_probe_mfma_sink_floats(void) { return (size_t)kBlocks * kThreads; }

extern "C" double cp_probe_mfma_flops(int32_t iters)
{
    // 32 x 32 x 16 multiply-adds per MFMA and wavefront
    return (double)kBlocks * (kThreads / 64) * (double)iters * kMfmaPerTrip * (2.0 * 32 * 32 * 16);
}

extern "C" int cp_probe_mfma(int32_t operands, int32_t iters, float *sink, void *stream)
{
    return launch(false, operands, iters, sink, stream);
}

extern "C" int cp_probe_mix(int32_t operands, int32_t iters, float *sink, void *stream)
{
    return launch(true, operands, iters, sink, stream);
}

extern "C" int cp_probe_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src) return -1;
    if (bytes == 0 || bytes % 16 != 0 || (uintptr_t)dst % 16 != 0 || (uintptr_t)src % 16 != 0) return -2;
    const size_t n = bytes / 16;
    const size_t per_block = 256 * kCopyUnroll;
    const unsigned blocks = (unsigned)std::min<size_t>((n + per_block - 1) / per_block, 256u * 16u);
    hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (u32x4 *)dst, (const u32x4 *)src, n);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

extern "C" int cp_probe_fill_lds(uint32_t pattern, void *stream)
{
    static std::once_flag once;
    static hipError_t attr = hipSuccess;
    std::call_once(once, [] {
        attr = hipFuncSetAttribute((const void *)fill_lds_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   kLdsFillBytes);
    });
    if (attr != hipSuccess) return -4;
    hipLaunchKernelGGL(fill_lds_kernel, dim3(kBlocks * 8), dim3(1024), kLdsFillBytes, (hipStream_t)stream, pattern,
                       (unsigned *)nullptr);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}
