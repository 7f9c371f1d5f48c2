/*
 * cp_extend: prefix-cached "extend" prefill attention over a paged KV cache (C ABI).
 *
 * Setting (paper, Section 1 and Section 2.1): during prefill an inference engine computes
 * the K/V of a prompt; a prefix cache keeps the K/V of earlier prompts as blocks addressed by
 * block identifiers; a request whose prompt starts with a cached prefix computes only its
 * uncached suffix, reading the prefix K/V back from the cache, and stores the new K/V so that
 * later requests can reuse it.  Exact-prefix reuse does not change the result (Section 1), so
 * the operations below are plain causal scaled-dot-product attention and a cache append.
 *
 * Notation: B requests; request r has P_r cached prefix tokens and E_r extend (suffix) tokens;
 * T = sum_r E_r; cu[r] = E_0 + ... + E_{r-1}; Hq query heads, Hkv KV heads, G = Hq / Hkv;
 * D = head_dim; PS = page_size.
 *
 * Memory layouts (all dense; bf16 carried as raw 16-bit patterns):
 *   q, out         [T][Hq][D]    bf16   DEVICE   request r owns rows [cu[r], cu[r] + E_r)
 *   k_new, v_new   [T][Hkv][D]   bf16   DEVICE
 *   kv_pages       [num_pages][2][Hkv][PS][D] bf16 DEVICE  (index 0 = K, 1 = V); one
 *                  (page, K|V, head) slab is PS*D*2 contiguous bytes
 *   block_table    [B][max_pages_per_req] int32 DEVICE; entry i is the physical page that
 *                  holds tokens [i*PS, (i+1)*PS) of the request; entries at or beyond
 *                  ceil((P_r + E_r) / PS) are never read
 *   prefix_lens, extend_lens [B] int32 DEVICE, with identical HOST copies in cp_shape
 *
 * Ownership: the caller owns every buffer and the stream.  The library allocates no device
 * memory, never synchronises and never changes the current device; all work is enqueued on
 * `stream` (a hipStream_t passed as void*; NULL is the default stream).  q, out, k_new, v_new
 * and kv_pages must be 16-byte aligned (the kernels move them in 16-byte pieces), the int32
 * arrays 4-byte aligned; a pointer that is not is refused with CP_ERR_ALIGN.
 *
 * Errors: every entry point validates its host-visible arguments before any launch and
 * returns CP_OK or a negative code; nothing is enqueued when a code other than CP_OK or
 * CP_ERR_LAUNCH is returned.  Device-side contents (block_table entries inside
 * [0, num_pages), device lengths equal to the host copies) are not validated by default,
 * because that needs a wait for the stream: cp_check_tables does it on request, and in debug
 * mode (cp_set_debug_validate, the environment variable CP_DEBUG_VALIDATE=1, or a library built
 * with -DCP_DEBUG_VALIDATE) cp_extend_attention and cp_write_kv run the same check first and
 * launch nothing when it fails.
 */
#ifndef CP_EXTEND_H
#define CP_EXTEND_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CP_OK = 0,
    CP_ERR_NULL = -1,      /* a required pointer is NULL */
    CP_ERR_SHAPE = -2,     /* unsupported or inconsistent shape (see cp_shape) */
    CP_ERR_WORKSPACE = -3, /* workspace missing, too small or misaligned; or, for the entry point
                              without a workspace, a shape that needs more than the library holds */
    CP_ERR_LAUNCH = -4,    /* the HIP runtime reported an error */
    CP_ERR_ALIGN = -5,     /* a device pointer is not aligned as required */
    CP_ERR_TABLE = -6,     /* check: a block_table entry in use lies outside [0, num_pages) */
    CP_ERR_LENGTHS = -7    /* check: device prefix_lens / extend_lens differ from the host copies */
};

typedef struct cp_shape {
    int32_t batch;             /* B >= 1 */
    int32_t num_q_heads;       /* Hq >= 1 */
    int32_t num_kv_heads;      /* Hkv >= 1, Hq % Hkv == 0; q head h uses KV head h / (Hq/Hkv) */
    int32_t head_dim;          /* must be 128 */
    int32_t page_size;         /* must be 16 */
    int32_t num_pages;         /* pages in kv_pages, >= 1 */
    int32_t max_pages_per_req; /* row stride of block_table; >= ceil((P_r+E_r)/PS) for all r */
    int32_t total_extend;      /* T; must equal the sum of h_extend_lens */
    float softmax_scale;       /* multiplies q.k before the softmax; finite and > 0 */
    int32_t num_splits;        /* split-K factor over the keys: 0 = chosen by the library
                                  (which also picks the decode-shaped kernel when every request
                                  has G * E_r <= 64 rows per KV head), 1 = never split,
                                  2..64 = forced */
    const int32_t *h_prefix_lens; /* HOST, length B, each >= 0 */
    const int32_t *h_extend_lens; /* HOST, length B, each >= 0 */
} cp_shape;

/*
 * Bytes of device scratch that cp_extend_attention needs for this shape (0 when the keys
 * are not split).  A pure function of *shape, including the host length arrays.  Returns 0
 * for an invalid shape (cp_extend_attention then reports the error).
 */
size_t cp_workspace_bytes(const cp_shape *shape);

/* The number of key ranges whose partial results cp_extend_attention will merge for this shape
 * (1 = no split; up to 64 when forced, up to 256 when chosen by the library; 0 if invalid). */
int32_t cp_num_splits(const cp_shape *shape);

/*
 * Which kernels cp_extend_attention will launch for this shape (launch planning is host integer
 * work on the lengths of the batch, the counterpart of the paper's host-side scheduling,
 * Section 5.2): a pure function of *shape.
 */
enum {
    CP_PLAN_INVALID = 0,
    CP_PLAN_ROW_TILED = 1,       /* extend_attn_kernel, keys not split */
    CP_PLAN_ROW_TILED_SPLIT = 2, /* extend_attn_kernel over key ranges + merge_splits_kernel */
    CP_PLAN_DECODE = 3           /* decode_attn_kernel (a wavefront per key chunk) + merge_splits_kernel */
};
int32_t cp_plan_kind(const cp_shape *shape);

/*
 * Extend attention (paper, Section 1: prefill over a prefix cache).  For request r, q head h,
 * g = h / G and extend row i in [0, E_r):
 *     key(j), val(j):  j <  P_r -> row j % PS of head g in page block_table[r][j / PS]
 *                      j >= P_r -> row cu[r] + j - P_r of k_new / v_new, head g
 *     s_j = softmax_scale * <q[cu[r]+i, h, :], key(j)>       for j = 0 .. P_r + i
 *     out[cu[r]+i, h, :] = sum_j softmax(s)_j * val(j)
 * Products are bf16 x bf16 accumulated in fp32, the softmax is fp32, out is rounded to bf16
 * (nearest even).  The row-tiled kernel first multiplies each query element by
 * softmax_scale * log2(e) and rounds it to bf16 (nearest even), so that the products are the
 * exponents of 2 directly: the result is the attention of a query that differs from the given
 * one by at most half a bf16 unit in the last place per element, i.e. by no more than the
 * rounding the query already carries; the decode-shaped kernel scales the fp32 scores instead.
 * The suffix K/V is read from k_new / v_new, never from kv_pages, so the
 * result does not depend on whether cp_write_kv ran before, after or not at all.  kv_pages is
 * only read.  Results are bitwise reproducible for a fixed shape (no atomics).
 *
 * workspace: DEVICE scratch of at least cp_workspace_bytes(shape) bytes, 256-byte aligned;
 * may be NULL when that size is 0.  Its contents are undefined afterwards.
 * Requests with E_r = 0 produce no rows.  Asynchronous on `stream`.
 */
int cp_extend_attention(const void *q, const void *k_new, const void *v_new,
                        const void *kv_pages, const int32_t *block_table,
                        const int32_t *prefix_lens, const int32_t *extend_lens, void *out,
                        void *stream, const cp_shape *shape, void *workspace,
                        size_t workspace_bytes);

/*
 * cp_extend_attention for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, result and checks as cp_extend_attention without the last two; the split-K /
 * decode partial results go to an array of cp_noalloc_scratch_bytes() bytes (64 MiB) that lives
 * inside the library, once per device, from the moment the library is loaded until the process
 * ends.  A shape whose cp_workspace_bytes exceeds that size is refused with CP_ERR_WORKSPACE
 * and nothing is launched.  The call allocates nothing and frees nothing (the array's device
 * address is looked up on the first call on each device).  All calls on one device share the
 * array: two such calls that overlap in time (different streams, different host threads) race
 * on it and must be serialised by the caller; calls on one stream are ordered and safe.
 */
int cp_extend_attention_noalloc(const void *q, const void *k_new, const void *v_new,
                                const void *kv_pages, const int32_t *block_table,
                                const int32_t *prefix_lens, const int32_t *extend_lens,
                                void *out, void *stream, const cp_shape *shape);

/* Size in bytes of the array behind cp_extend_attention_noalloc: its largest workspace. */
size_t cp_noalloc_scratch_bytes(void);

/*
 * Cache append (paper, Section 1: the prefix cache stores the K/V of prior prompts).  For
 * request r, row j < E_r and KV head g, the bit patterns of k_new[cu[r]+j, g, :] and
 * v_new[cu[r]+j, g, :] are copied to page block_table[r][(P_r+j) / PS], slot (P_r+j) % PS.
 * No other element of kv_pages is touched.  Two rows that map to the same destination slot
 * (overlapping page lists of different requests) give an undefined winner.
 * Asynchronous on `stream`.
 */
int cp_write_kv(const void *k_new, const void *v_new, void *kv_pages,
                const int32_t *block_table, const int32_t *prefix_lens,
                const int32_t *extend_lens, void *stream, const cp_shape *shape);

/*
 * Check of the device-side contents that the two calls above trust (the setting is the same:
 * paper, Section 2.1, a prefix cache maps prompts to KV-block identifiers, and a wrong
 * identifier would make the kernels read or write outside the page pool).  Copies the device
 * prefix_lens / extend_lens to the host and compares them with the host copies in *shape
 * (CP_ERR_LENGTHS), then runs a small kernel that reads block_table[r][i] for every slot in use,
 * i < ceil((P_r + E_r) / PS), and reports the first entry outside [0, num_pages) (CP_ERR_TABLE);
 * no page is dereferenced.  WAITS for `stream`; meant for tests and debugging.
 * info: optional HOST int32[3]; on CP_ERR_TABLE {request, slot, entry}, on CP_ERR_LENGTHS
 * {request, device P_r, device E_r}, otherwise -1.
 */
int cp_check_tables(const int32_t *block_table, const int32_t *prefix_lens,
                    const int32_t *extend_lens, void *stream, const cp_shape *shape,
                    int32_t *info);

/* Debug mode on (non-zero) or off for this process: see "Errors" at the top. */
void cp_set_debug_validate(int on);

/* Static, human-readable text for a status code. */
const char *cp_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* CP_EXTEND_H */
