// cp_probe: measurement aids behind the C ABI of cp_probe.h.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cp_probe.h"

namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kBlocks = 512;  // two workgroups of four wavefronts per compute unit
constexpr int kThreads = 256;
constexpr int kMfmaPerTrip = 8;

__device__ inline unsigned mix(unsigned x)
{
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}
// two bf16 with random sign and mantissa and the exponent of 1.0
__device__ inline unsigned random_pair(unsigned seed) { return (mix(seed) & 0x807f807fu) | 0x3f803f80u; }

// Eight independent accumulator tiles per wavefront, so that consecutive MFMAs never wait for
// each other; the B operand rotates so that the loop cannot be folded.
template <bool kRandom>
__global__ __launch_bounds__(kThreads) void mfma_stream_kernel(float *sink, int iters)
{
    f32x16 acc[kMfmaPerTrip];
    u32x4 a[kMfmaPerTrip], b[kMfmaPerTrip];
#pragma unroll
    for (int i = 0; i < kMfmaPerTrip; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const unsigned seed = (blockIdx.x * kThreads + threadIdx.x) * 64u + i * 8u + e;
            a[i][e] = kRandom ? random_pair(seed) : 0x3f803f80u;
            b[i][e] = kRandom ? random_pair(seed + 4u) : 0x3f803f80u;
        }
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kMfmaPerTrip; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]),
                                                             __builtin_bit_cast(bf16x8, b[(i + it) & 7]), acc[i],
                                                             0, 0, 0);
    }
    float r = 0.f;
#pragma unroll
    for (int i = 0; i < kMfmaPerTrip; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) r += acc[i][v];
    sink[blockIdx.x * kThreads + threadIdx.x] = r;
}

} // namespace

extern "C" size_t cp_probe_mfma_sink_floats(void) { return (size_t)kBlocks * kThreads; }

extern "C" double cp_probe_mfma_flops(int32_t iters)
{
    // 32 x 32 x 16 multiply-adds per MFMA and wavefront
    return (double)kBlocks * (kThreads / 64) * (double)iters * kMfmaPerTrip * (2.0 * 32 * 32 * 16);
}

extern "C" int cp_probe_mfma(int32_t random_operands, int32_t iters, float *sink, void *stream)
{
    if (!sink) return -1;
    if (iters < 1 || iters > (1 << 24)) return -2;
    hipStream_t hs = (hipStream_t)stream;
    if (random_operands) hipLaunchKernelGGL(mfma_stream_kernel<true>, dim3(kBlocks), dim3(kThreads), 0, hs, sink, iters);
    else hipLaunchKernelGGL(mfma_stream_kernel<false>, dim3(kBlocks), dim3(kThreads), 0, hs, sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}
