// cp_context_dedup: multi-turn context de-duplication behind the C ABI of cp_context_dedup.h
// (paper, Section 6 and the appendix algorithm "Context De-duplication").  Plain C++; no GPU call.
#include <stdint.h>

#include <new>
#include <unordered_map>
#include <unordered_set>
#include <vector>

#include "cp_context_dedup.h"

namespace {

inline uint64_t fnv1a(const uint8_t *p, int64_t len)
{
    uint64_t h = 0xcbf29ce484222325ull;
    for (int64_t i = 0; i < len; ++i) {
        h ^= p[i];
        h *= 0x100000001b3ull;
    }
    return h;
}

// End offsets of the sub-blocks of bytes[0, len): after every line whose hash (without the
// newline) is 0 modulo `modulus`, and at the end.
void chunk_ends(const uint8_t *bytes, int64_t len, uint64_t modulus, std::vector<int64_t> &ends)
{
    ends.clear();
    int64_t line_start = 0, sub_start = 0;
    for (int64_t i = 0; i < len; ++i) {
        if (bytes[i] != '\n') continue;
        if (fnv1a(bytes + line_start, i - line_start) % modulus == 0) {
            ends.push_back(i + 1);
            sub_start = i + 1;
        }
        line_start = i + 1;
    }
    // a last line without a newline is tested like any other; what is left over ends the block
    if (line_start < len && fnv1a(bytes + line_start, len - line_start) % modulus == 0) {
        ends.push_back(len);
        sub_start = len;
    }
    if (sub_start < len) ends.push_back(len);
}

} // namespace

// State of one conversation: which blocks earlier turns brought, and for every sub-block content
// (by hash) the block that brought it first.
struct cp_dedup {
    uint64_t modulus = 1;
    std::unordered_set<int32_t> earlier_turn_blocks;
    std::unordered_map<uint64_t, int32_t> owner_of_hash;
};

extern "C" uint64_t cp_dedup_hash(const uint8_t *bytes, int64_t len)
{
    return (bytes && len > 0) ? fnv1a(bytes, len) : 0xcbf29ce484222325ull;
}

extern "C" int cp_dedup_chunks(const uint8_t *bytes, int64_t len, uint64_t modulus, int64_t *ends, int32_t cap,
                               int32_t *count)
{
    if (!count || (len > 0 && !bytes)) return -1;
    if (len < 0 || modulus < 1 || cap < 0) return -2;
    std::vector<int64_t> e;
    chunk_ends(bytes, len, modulus, e);
    *count = (int32_t)e.size();
    if ((int32_t)e.size() > cap) return -2;
    if (!e.empty() && !ends) return -1;
    for (size_t i = 0; i < e.size(); ++i) ends[i] = e[i];
    return 0;
}

extern "C" int cp_dedup_create(uint64_t modulus, cp_dedup **out)
{
    if (!out) return -1;
    *out = nullptr;
    if (modulus < 1) return -2;
    cp_dedup *c = new (std::nothrow) cp_dedup();
    if (!c) return -2;
    c->modulus = modulus;
    *out = c;
    return 0;
}

extern "C" void cp_dedup_free(cp_dedup *conv) { delete conv; }

extern "C" int cp_dedup_turn(cp_dedup *conv, const int32_t *ids, const uint8_t *bytes, const int64_t *offsets,
                             int32_t n, int32_t *block_ref, cp_dedup_sub *subs, int32_t subs_cap,
                             int32_t *subs_count, int64_t *kept_bytes)
{
    if (!conv || !subs_count) return -1;
    if (n < 0 || subs_cap < 0) return -2;
    if (n > 0 && (!ids || !offsets || !block_ref)) return -1;
    for (int32_t i = 0; i < n; ++i)
        if (offsets[i] < 0 || offsets[i + 1] < offsets[i]) return -2;
    if (n > 0 && offsets[n] > 0 && !bytes) return -1;

    // Pass over whole blocks: a block that an earlier turn of the conversation brought is
    // answered by a reference and not looked into.
    std::vector<int32_t> to_cut;
    for (int32_t i = 0; i < n; ++i) {
        block_ref[i] = conv->earlier_turn_blocks.count(ids[i]) ? 1 : 0;
        if (!block_ref[i]) to_cut.push_back(i);
    }
    // Pass over the sub-blocks of the others, in order: content that a different block owns
    // becomes a reference to that block, anything else is kept and owned from now on.  The
    // ownership table is edited on a copy, so that a too small output buffer leaves the
    // conversation as it was.
    std::unordered_map<uint64_t, int32_t> owners = conv->owner_of_hash;
    std::vector<cp_dedup_sub> out;
    std::vector<int64_t> ends;
    int64_t kept = 0;
    for (int32_t i : to_cut) {
        const uint8_t *text = bytes + offsets[i];
        chunk_ends(text, offsets[i + 1] - offsets[i], conv->modulus, ends);
        int64_t begin = 0;
        for (int64_t end : ends) {
            const auto claim = owners.emplace(fnv1a(text + begin, end - begin), ids[i]);
            const int32_t owner = claim.first->second; // this block itself when the content is new
            out.push_back(cp_dedup_sub{i, owner == ids[i] ? -1 : owner, begin, end});
            if (owner == ids[i]) kept += end - begin;
            begin = end;
        }
    }
    *subs_count = (int32_t)out.size();
    if ((int32_t)out.size() > subs_cap) return -2;
    if (!out.empty() && !subs) return -1;
    for (size_t k = 0; k < out.size(); ++k) subs[k] = out[k];
    conv->owner_of_hash.swap(owners);
    conv->earlier_turn_blocks.insert(ids, ids + n);
    if (kept_bytes) *kept_bytes = kept;
    return 0;
}
