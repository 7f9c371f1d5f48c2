/*
 * cp_context_distance: pairwise distance between contexts for the context index (C ABI).
 *
 * The paper builds its context index by hierarchical clustering over pairwise context
 * distances (Section 4.1, "Index creation"; first phase of the appendix algorithm "Context Index
 * Construction via Hierarchical Clustering", which the paper runs on a GPU or on CPUs) with the
 * distance of Eq. 1:
 *
 *     d_ij = 1 - |S_ij| / max(|C_i|, |C_j|) + alpha * (sum_{k in S_ij} |p_i(k) - p_j(k)|) / |S_ij|
 *
 * A context C_i is an ordered list of distinct context-block ids, S_ij the ids present in both
 * contexts and p_i(k) the 0-based position of id k in C_i.  Where nothing is shared the last
 * term is taken as 0 (d = 1); two empty contexts are at distance 0.
 *
 * This entry point fills the whole n x n matrix (symmetric, zero diagonal).
 */
#ifndef CP_CONTEXT_DISTANCE_H
#define CP_CONTEXT_DISTANCE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * contexts  DEVICE [n][stride] int32, row i holds lens[i] block ids >= 0, distinct within the
 *           row, in rank order; the rest of the row is ignored.  16-byte aligned.
 * lens      DEVICE [n] int32, 0 <= lens[i] <= stride (not validated: it lives on the device)
 * n         number of contexts, 0 <= n <= 65536
 * stride    ints per row, 1 <= stride <= 32, and a multiple of 4
 * alpha     weight of the positional term, finite and >= 0 (the paper uses 0.001 .. 0.01)
 * dist      DEVICE [n][n] float32, written completely; caller-owned
 * stream    hipStream_t as void*, NULL = default stream
 *
 * Arithmetic: set intersection and position gaps are exact integers; the three terms are
 * combined in fp32.  Asynchronous on `stream`; allocates nothing; never synchronises.
 * Returns 0 on success, -1 for a NULL pointer (with n > 0), -2 for an argument out of range,
 * -4 if the HIP runtime reported a launch error.  Nothing is launched on -1 / -2.
 */
int cp_context_distance(const int32_t *contexts, const int32_t *lens, int32_t n, int32_t stride,
                        float alpha, float *dist, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CP_CONTEXT_DISTANCE_H */
