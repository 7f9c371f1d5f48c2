/*
 * CPU oracle for the pairwise context distance of the paper's context index (Section 4.1,
 * Eq. 1).  TEST INFRASTRUCTURE ONLY: shares no code with the GPU library and is called only by
 * the tests, the smoke check and the CPU-baseline leg of the benchmark.
 *
 * A context C_i is an ordered list of distinct context-block ids (retrieval rank order).  For
 * two contexts, S_ij is the set of ids present in both and p_i(k) the position of id k in C_i:
 *
 *     d_ij = 1 - |S_ij| / max(|C_i|, |C_j|) + alpha * ( sum_{k in S_ij} |p_i(k) - p_j(k)| ) / |S_ij|
 *
 * The paper does not say what the last term is when nothing is shared (0/0): it is taken as 0,
 * so disjoint contexts are at distance 1.  Two empty contexts are at distance 0.
 *
 * contexts: [n][stride] int32, row i holds lens[i] ids; dist: [n][n] double.
 */
#include <stdint.h>
#include <stdlib.h>

int oracle_context_distance(const int32_t *contexts, const int32_t *lens, int32_t n,
                            int32_t stride, double alpha, double *dist)
{
    if (n < 0 || stride < 0) return -1;
    for (int32_t i = 0; i < n; ++i)
        if (lens[i] < 0 || lens[i] > stride) return -1;
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < n; ++i) {
        const int32_t *ci = contexts + (int64_t)i * stride;
        for (int32_t j = 0; j < n; ++j) {
            const int32_t *cj = contexts + (int64_t)j * stride;
            int shared = 0;
            long gap = 0;
            for (int32_t a = 0; a < lens[i]; ++a) {
                for (int32_t b = 0; b < lens[j]; ++b) {
                    if (ci[a] == cj[b]) {
                        ++shared;
                        gap += labs((long)a - (long)b);
                        break; /* ids are distinct inside a context */
                    }
                }
            }
            int longest = lens[i] > lens[j] ? lens[i] : lens[j];
            double d;
            if (longest == 0) d = 0.0;
            else if (shared == 0) d = 1.0;
            else d = 1.0 - (double)shared / (double)longest + alpha * ((double)gap / (double)shared);
            dist[(int64_t)i * n + j] = d;
        }
    }
    return 0;
}
