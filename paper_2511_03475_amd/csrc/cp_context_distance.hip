// Pairwise context distance (paper, Section 4.1, Eq. 1) for gfx950.
//
// Integer set-intersection work bound by the vector ALU, no matrix cores.  One thread owns
// one column context C_j, held in registers; the workgroup walks over a strip of row contexts
// C_i whose ids are wave-uniform and therefore sit in scalar registers, so the inner loop is one
// compare (SGPR id against VGPR id) and one conditional move per (a, b) pair of positions, and
// the 256 threads of a workgroup write 256 consecutive floats of a row of the matrix.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cp_context_distance.h"

namespace {

constexpr int kThreads = 256; // columns per workgroup
constexpr int kRowsPerBlock = 64;

template <int kMax>
__global__ __launch_bounds__(kThreads) void context_distance_kernel(const int32_t *__restrict__ contexts,
                                                                   const int32_t *__restrict__ lens,
                                                                   int n, int stride, float alpha,
                                                                   float *__restrict__ dist)
{
    const int j = blockIdx.x * kThreads + threadIdx.x;
    const bool col_ok = j < n;
    const int jc = col_ok ? j : n - 1;
    // column context in registers; unused slots can never match (row ids are >= 0 or -2)
    const int len_j = lens[jc];
    int cj[kMax];
#pragma unroll
    for (int b = 0; b < kMax; ++b) {
        const int id = (b < stride) ? contexts[(int64_t)jc * stride + b] : -1;
        cj[b] = (b < len_j) ? id : -1;
    }
    const int i0 = blockIdx.y * kRowsPerBlock;
    const int i1 = min(n, i0 + kRowsPerBlock);
    for (int i = i0; i < i1; ++i) {
        const int len_i = lens[i]; // uniform: scalar load
        const int32_t *ci = contexts + (int64_t)i * stride;
        int shared = 0, gap = 0;
#pragma unroll
        for (int a = 0; a < kMax; ++a) {
            if (a < stride) {
                const int id = (a < len_i) ? ci[a] : -2; // uniform
                int hit = 0;                             // position + 1 of id in C_j, 0 if absent
#pragma unroll
                for (int b = 0; b < kMax; ++b) hit = (cj[b] == id) ? (b + 1) : hit;
                shared += hit != 0;
                gap += hit != 0 ? abs(a + 1 - hit) : 0;
            }
        }
        const int longest = max(len_i, len_j);
        float d;
        if (longest == 0) d = 0.f;
        else if (shared == 0) d = 1.f;
        else d = 1.f - (float)shared / (float)longest + alpha * ((float)gap / (float)shared);
        if (col_ok) dist[(int64_t)i * n + j] = d;
    }
}

} // namespace

extern "C" int cp_context_distance(const int32_t *contexts, const int32_t *lens, int32_t n,
                                   int32_t stride, float alpha, float *dist, void *stream)
{
    if (n < 0 || n > 65536 || stride < 1 || stride > 32 || stride % 4 != 0) return -2;
    if (!(alpha >= 0.f) || !(alpha < 3.0e38f)) return -2;
    if (n == 0) return 0;
    if (!contexts || !lens || !dist) return -1;
    const dim3 grid((unsigned)((n + kThreads - 1) / kThreads), (unsigned)((n + kRowsPerBlock - 1) / kRowsPerBlock));
    hipStream_t hs = static_cast<hipStream_t>(stream);
    if (stride <= 16)
        hipLaunchKernelGGL(context_distance_kernel<16>, grid, dim3(kThreads), 0, hs, contexts, lens, n, stride,
                           alpha, dist);
    else
        hipLaunchKernelGGL(context_distance_kernel<32>, grid, dim3(kThreads), 0, hs, contexts, lens, n, stride,
                           alpha, dist);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}
