/*
 * cp_context_dedup: the paper's context de-duplication for multi-turn conversations (C ABI).
 *
 * Paper, Section 6 and the appendix algorithm "Context De-duplication".  Per conversation the
 * library remembers (a) the ids of the context blocks of earlier turns and (b) for every
 * sub-block hash the block it was first seen in.  A turn brings new context blocks (id + text):
 *   - a block whose id was seen in an earlier turn is replaced as a whole by a reference to it;
 *   - any other block is cut into sub-blocks by content-defined chunking over its text lines (a
 *     sub-block ends after every line whose hash is 0 modulo the chunk modulus M, and at the end
 *     of the block); a sub-block whose hash is already known under ANOTHER block's id is replaced
 *     by a reference to that block, otherwise it is kept and recorded under this block's id;
 *   - after the whole turn its block ids join the seen set.
 * The library reports which byte ranges are kept and which are replaced by a reference to which
 * block; wording the annotations is the caller's business.
 *
 * Choices the paper leaves open, as taken here: Hash is 64-bit FNV-1a over bytes, for lines
 * (without their newline) and for sub-blocks (all their bytes); a line runs up to and including
 * its newline, the last one may lack it.
 *
 * Host memory only; no GPU call.  Returns 0 on success, -1 for a NULL pointer, -2 for an argument
 * out of range (including an output buffer that is too small: the needed count is still stored,
 * and the conversation state is then left unchanged).  A handle is not thread-safe.
 */
#ifndef CP_CONTEXT_DEDUP_H
#define CP_CONTEXT_DEDUP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cp_dedup cp_dedup;

typedef struct cp_dedup_sub {
    int32_t block;  /* position of the block in this turn's list */
    int32_t ref;    /* id of the block this sub-block is replaced by a reference to; -1 = kept */
    int64_t begin;  /* byte range inside the block's text */
    int64_t end;
} cp_dedup_sub;

/* 64-bit FNV-1a of len bytes (offset basis 0xcbf29ce484222325, prime 0x100000001b3). */
uint64_t cp_dedup_hash(const uint8_t *bytes, int64_t len);

/*
 * Content-defined chunking of one block: ends[k] is the end offset of sub-block k (the last is
 * len).  modulus >= 1.  count receives the number of sub-blocks (0 for an empty block).
 */
int cp_dedup_chunks(const uint8_t *bytes, int64_t len, uint64_t modulus, int64_t *ends,
                    int32_t cap, int32_t *count);

/* A new conversation with chunk modulus M >= 1. */
int cp_dedup_create(uint64_t modulus, cp_dedup **out);
void cp_dedup_free(cp_dedup *conv);

/*
 * One turn.
 * ids        HOST [n] int32 block ids of the new context, in order
 * bytes      HOST the texts of the n blocks, concatenated
 * offsets    HOST [n + 1] int64, block i is bytes[offsets[i] .. offsets[i+1]); non-decreasing
 * block_ref  HOST [n] int32 out: 1 = the whole block is replaced by a reference to its earlier
 *            occurrence, 0 = processed sub-block by sub-block
 * subs       HOST [subs_cap] out: the sub-blocks of all processed blocks, in order
 * subs_count out: number of entries written (or needed, with -2)
 * kept_bytes out (may be NULL): bytes of this turn that still have to be prefilled
 */
int cp_dedup_turn(cp_dedup *conv, const int32_t *ids, const uint8_t *bytes, const int64_t *offsets,
                  int32_t n, int32_t *block_ref, cp_dedup_sub *subs, int32_t subs_cap,
                  int32_t *subs_count, int64_t *kept_bytes);

#ifdef __cplusplus
}
#endif
#endif /* CP_CONTEXT_DEDUP_H */
