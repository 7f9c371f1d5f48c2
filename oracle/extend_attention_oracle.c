/*
 * CPU oracle for prefix-cached "extend" prefill attention over a paged KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition that the
 * GPU library is checked against.  It shares no code with the GPU path, and nothing
 * in the product may call it: only the tests, the smoke check and the CPU-baseline leg
 * of the benchmark do.
 *
 * What it computes.  The paper (Section 1; Section 2.1) describes the setting: during
 * prefill an engine computes K/V for the prompt, a prefix cache keeps the K/V of earlier
 * prompts as blocks addressed by identifiers, and a request whose prompt starts with a
 * cached prefix only computes its uncached suffix.  Exact-prefix reuse leaves the result
 * unchanged (Section 1: exact prefix matching preserves accuracy), so the result is
 * plain causal scaled-dot-product attention of the suffix rows over prefix + suffix keys.
 * The paper never writes the attention formula down; it is the textbook one:
 *
 *   request r, q head h, KV head g = h / (Hq / Hkv), extend row i in [0, E_r):
 *     key(j), val(j), j in [0, P_r + E_r):
 *        j <  P_r : row (j % PS) of head g in page block_table[r][j / PS]
 *        j >= P_r : row cu[r] + (j - P_r) of k_new / v_new, head g
 *     s_j = scale * sum_d q[cu[r]+i, h, d] * key(j)[d]      for j in [0, P_r + i]
 *     out[cu[r]+i, h, :] = sum_j softmax(s)_j * val(j)
 *
 * All inputs are bf16 bit patterns widened exactly to double; every sum, the exponential
 * and the division are double.  No blocking, no fusion, no reordering: one row at a time,
 * scores first, then max, then exponentials, then the weighted sum.
 *
 * Layouts (dense, row-major):
 *   q, out          [T][Hq][D]          T = sum_r E_r, cu = exclusive prefix sum of E
 *   k_new, v_new    [T][Hkv][D]
 *   kv_pages        [num_pages][2][Hkv][PS][D]     index 0 = K, 1 = V
 *   block_table     [B][max_pages_per_req]
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Pointer to the D elements of key (which = 0) or value (which = 1) number j of request r. */
static const uint16_t *kv_row(const uint16_t *k_new, const uint16_t *v_new,
                              const uint16_t *kv_pages, const int32_t *table_row,
                              int64_t cu_r, int32_t P, int32_t Hkv, int32_t D, int32_t PS,
                              int32_t g, int64_t j, int which)
{
    if (j < P) {
        int64_t page = table_row[j / PS];
        int64_t slot = j % PS;
        return kv_pages + ((((page * 2 + which) * Hkv + g) * PS + slot) * (int64_t)D);
    }
    const uint16_t *src = which ? v_new : k_new;
    return src + ((cu_r + (j - P)) * Hkv + g) * (int64_t)D;
}

/*
 * Attention of one (row, head) over the visible keys restricted to [key_lo, key_hi).
 * Writes D outputs; returns log(sum_j exp(s_j)) over the keys used (-inf if none,
 * in which case the outputs are zero).
 */
static double attend_row(const uint16_t *qrow, const uint16_t *k_new, const uint16_t *v_new,
                         const uint16_t *kv_pages, const int32_t *table_row, int64_t cu_r,
                         int32_t P, int32_t Hkv, int32_t D, int32_t PS, int32_t g,
                         int64_t key_lo, int64_t key_hi, double scale, double *scores,
                         double *out)
{
    int64_t n = key_hi - key_lo;
    for (int d = 0; d < D; ++d) out[d] = 0.0;
    if (n <= 0) return -INFINITY;
    double m = -INFINITY;
    for (int64_t t = 0; t < n; ++t) {
        const uint16_t *k = kv_row(k_new, v_new, kv_pages, table_row, cu_r, P, Hkv, D, PS, g,
                                   key_lo + t, 0);
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += bf16_to_double(qrow[d]) * bf16_to_double(k[d]);
        scores[t] = scale * dot;
        if (scores[t] > m) m = scores[t];
    }
    double denom = 0.0;
    for (int64_t t = 0; t < n; ++t) {
        scores[t] = exp(scores[t] - m);
        denom += scores[t];
    }
    for (int64_t t = 0; t < n; ++t) {
        const uint16_t *v = kv_row(k_new, v_new, kv_pages, table_row, cu_r, P, Hkv, D, PS, g,
                                   key_lo + t, 1);
        double w = scores[t] / denom;
        for (int d = 0; d < D; ++d) out[d] += w * bf16_to_double(v[d]);
    }
    return m + log(denom);
}

/*
 * rows: packed row indices in [0, T) to compute, or NULL for all T rows (n_rows = T).
 * key_lo / key_hi: restrict the keys of every row to [key_lo, key_hi) intersected with the
 *   causal range [0, P_r + i]; pass 0 and a negative key_hi for "no restriction".
 * out: [n_rows][Hq][D] double.  lse: optional [n_rows][Hq] log-sum-exp of the scores used.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int oracle_extend_attention(const uint16_t *q, const uint16_t *k_new, const uint16_t *v_new,
                            const uint16_t *kv_pages, const int32_t *block_table,
                            const int32_t *prefix_lens, const int32_t *extend_lens,
                            int32_t batch, int32_t Hq, int32_t Hkv, int32_t D, int32_t PS,
                            int32_t max_pages_per_req, double scale, const int32_t *rows,
                            int64_t n_rows, int64_t key_lo, int64_t key_hi, double *out,
                            double *lse)
{
    if (batch <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || D <= 0 || PS <= 0) return -1;
    int64_t *cu = (int64_t *)malloc((size_t)(batch + 1) * sizeof(int64_t));
    if (!cu) return -1;
    cu[0] = 0;
    int64_t max_n = 0;
    for (int r = 0; r < batch; ++r) {
        if (prefix_lens[r] < 0 || extend_lens[r] < 0) { free(cu); return -1; }
        cu[r + 1] = cu[r] + extend_lens[r];
        int64_t n = (int64_t)prefix_lens[r] + extend_lens[r];
        if (n > max_n) max_n = n;
    }
    int64_t T = cu[batch];
    if (!rows) n_rows = T;
    int G = Hq / Hkv;
    int failed = 0;
#pragma omp parallel
    {
        double *scores = (double *)malloc((size_t)(max_n > 0 ? max_n : 1) * sizeof(double));
        if (!scores) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for collapse(2) schedule(dynamic, 1)
            for (int64_t s = 0; s < n_rows; ++s) {
                for (int h = 0; h < Hq; ++h) {
                    int64_t row = rows ? rows[s] : s;
                    int r = 0;
                    while (r + 1 < batch && row >= cu[r + 1]) ++r;
                    int64_t i = row - cu[r];
                    int32_t P = prefix_lens[r];
                    int64_t hi = (int64_t)P + i + 1; /* keys 0 .. P+i inclusive */
                    int64_t lo = key_lo > 0 ? key_lo : 0;
                    if (key_hi >= 0 && key_hi < hi) hi = key_hi;
                    double l = attend_row(q + (row * Hq + h) * (int64_t)D, k_new, v_new, kv_pages,
                                          block_table + (int64_t)r * max_pages_per_req, cu[r], P,
                                          Hkv, D, PS, h / G, lo, hi, scale, scores,
                                          out + (s * Hq + h) * (int64_t)D);
                    if (lse) lse[s * Hq + h] = l;
                }
            }
        }
        free(scores);
    }
    free(cu);
    return failed ? -1 : 0;
}

/*
 * Cache append: for request r, extend row j < E_r and KV head g, the 16-bit patterns of
 * k_new[cu[r]+j, g, :] and v_new[cu[r]+j, g, :] go to page block_table[r][(P_r+j)/PS],
 * slot (P_r+j) % PS.  Every other element of kv_pages keeps its value.
 */
int oracle_write_kv(const uint16_t *k_new, const uint16_t *v_new, uint16_t *kv_pages,
                    const int32_t *block_table, const int32_t *prefix_lens,
                    const int32_t *extend_lens, int32_t batch, int32_t Hkv, int32_t D,
                    int32_t PS, int32_t max_pages_per_req)
{
    if (batch <= 0 || Hkv <= 0 || D <= 0 || PS <= 0) return -1;
    int64_t cu = 0;
    for (int r = 0; r < batch; ++r) {
        const int32_t *table_row = block_table + (int64_t)r * max_pages_per_req;
        for (int64_t j = 0; j < extend_lens[r]; ++j) {
            int64_t tok = (int64_t)prefix_lens[r] + j;
            int64_t page = table_row[tok / PS];
            int64_t slot = tok % PS;
            for (int g = 0; g < Hkv; ++g) {
                const uint16_t *ks = k_new + ((cu + j) * Hkv + g) * (int64_t)D;
                const uint16_t *vs = v_new + ((cu + j) * Hkv + g) * (int64_t)D;
                uint16_t *kd = kv_pages + ((((page * 2 + 0) * Hkv + g) * PS + slot) * (int64_t)D);
                uint16_t *vd = kv_pages + ((((page * 2 + 1) * Hkv + g) * PS + slot) * (int64_t)D);
                memcpy(kd, ks, (size_t)D * sizeof(uint16_t));
                memcpy(vd, vs, (size_t)D * sizeof(uint16_t));
            }
        }
        cu += extend_lens[r];
    }
    return 0;
}
