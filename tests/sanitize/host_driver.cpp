// Driver for the address / undefined-behaviour sanitizer build of the CPU-only code: the fp64
// oracle (C) and the two host libraries (context index, context de-duplication).  Every call is
// made on small seeded inputs, including the error paths; the sanitizers abort on the first
// finding, so exit status 0 means none.  Values are checked only loosely here (the pytest suites
// check them); what matters is that every access stays inside its buffers.
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <string>
#include <vector>

#include "cp_context_dedup.h"
#include "cp_context_index.h"

extern "C" {
int oracle_extend_attention(const uint16_t *q, const uint16_t *k_new, const uint16_t *v_new, const uint16_t *kv_pages,
                            const int32_t *block_table, const int32_t *prefix_lens, const int32_t *extend_lens,
                            int32_t batch, int32_t Hq, int32_t Hkv, int32_t D, int32_t PS, int32_t max_pages_per_req,
                            double scale, const int32_t *rows, int64_t n_rows, int64_t key_lo, int64_t key_hi,
                            double *out, double *lse);
int oracle_write_kv(const uint16_t *k_new, const uint16_t *v_new, uint16_t *kv_pages, const int32_t *block_table,
                    const int32_t *prefix_lens, const int32_t *extend_lens, int32_t batch, int32_t Hkv, int32_t D,
                    int32_t PS, int32_t max_pages_per_req);
int oracle_context_distance(const int32_t *contexts, const int32_t *lens, int32_t n, int32_t stride, double alpha,
                            double *dist);
}

#define CHECK(c)                                                                  \
    do {                                                                          \
        if (!(c)) {                                                               \
            fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #c); \
            exit(1);                                                              \
        }                                                                         \
    } while (0)

static uint32_t g_state = 12345u;
static uint32_t rnd() { g_state = g_state * 1664525u + 1013904223u; return g_state >> 8; }
static uint16_t rnd_bf16() // a value in (-2, 2) with a random mantissa
{
    const uint32_t r = rnd();
    return (uint16_t)(((r & 1u) << 15) | ((126u + (r >> 1) % 2u) << 7) | ((r >> 3) & 0x7fu));
}

static void attention_and_cache_write()
{
    const int B = 3, Hq = 4, Hkv = 2, D = 16, PS = 4;
    const int32_t P[B] = {5, 0, 9}, E[B] = {3, 6, 1};
    int T = 0, width = 0, pages = 0;
    for (int r = 0; r < B; ++r) {
        T += E[r];
        const int need = (P[r] + E[r] + PS - 1) / PS;
        width = need > width ? need : width;
        pages += need;
    }
    std::vector<int32_t> table((size_t)B * width, -1);
    int next = pages; // pages handed out from the top down, so the table is not the identity
    for (int r = 0; r < B; ++r)
        for (int i = 0; i < (P[r] + E[r] + PS - 1) / PS; ++i) table[(size_t)r * width + i] = --next;
    std::vector<uint16_t> q((size_t)T * Hq * D), k((size_t)T * Hkv * D), v(k.size()), pool((size_t)pages * 2 * Hkv * PS * D);
    for (auto &x : q) x = rnd_bf16();
    for (auto &x : k) x = rnd_bf16();
    for (auto &x : v) x = rnd_bf16();
    for (auto &x : pool) x = rnd_bf16();
    std::vector<double> out((size_t)T * Hq * D), lse((size_t)T * Hq);
    CHECK(oracle_extend_attention(q.data(), k.data(), v.data(), pool.data(), table.data(), P, E, B, Hq, Hkv, D, PS,
                                  width, 0.25, nullptr, T, 0, -1, out.data(), lse.data()) == 0);
    for (double x : out) CHECK(isfinite(x) && fabs(x) < 4.0);
    const int32_t rows[3] = {0, T - 1, 4};
    CHECK(oracle_extend_attention(q.data(), k.data(), v.data(), pool.data(), table.data(), P, E, B, Hq, Hkv, D, PS,
                                  width, 0.25, rows, 3, 2, 7, out.data(), nullptr) == 0);
    CHECK(oracle_extend_attention(q.data(), k.data(), v.data(), pool.data(), table.data(), P, E, B, 3, Hkv, D, PS,
                                  width, 0.25, nullptr, T, 0, -1, out.data(), nullptr) == -1);
    std::vector<uint16_t> before = pool;
    CHECK(oracle_write_kv(k.data(), v.data(), pool.data(), table.data(), P, E, B, Hkv, D, PS, width) == 0);
    size_t changed = 0;
    for (size_t i = 0; i < pool.size(); ++i) changed += pool[i] != before[i];
    CHECK(changed > 0 && changed <= (size_t)T * Hkv * D * 2);
}

static void distances_index_and_schedule()
{
    const int n = 40, stride = 8;
    std::vector<int32_t> C((size_t)n * stride, -1), L(n);
    for (int i = 0; i < n; ++i) {
        L[i] = 1 + (int32_t)(rnd() % stride);
        for (int a = 0; a < L[i]; ++a) {
            int32_t id;
            bool fresh;
            do {
                id = (int32_t)(rnd() % 20);
                fresh = true;
                for (int b = 0; b < a; ++b) fresh = fresh && C[(size_t)i * stride + b] != id;
            } while (!fresh);
            C[(size_t)i * stride + a] = id;
        }
    }
    memcpy(&C[(size_t)7 * stride], &C[(size_t)3 * stride], stride * sizeof(int32_t)); // a duplicate context
    L[7] = L[3];
    std::vector<double> dist((size_t)n * n);
    CHECK(oracle_context_distance(C.data(), L.data(), n, stride, 0.001, dist.data()) == 0);
    for (int i = 0; i < n; ++i) CHECK(dist[(size_t)i * n + i] == 0.0);

    std::vector<int32_t> first_of(n);
    int32_t m = 0;
    CHECK(cp_index_distinct(C.data(), L.data(), n, stride, first_of.data(), &m) == 0);
    CHECK(m > 0 && m < n && first_of[7] == first_of[3]);
    cp_index *idx = nullptr;
    CHECK(cp_index_build(C.data(), L.data(), n, stride, 0.001, nullptr, 0, &idx) == 0 && idx);
    CHECK(cp_index_num_contexts(idx) == n);
    const int32_t nodes = cp_index_num_nodes(idx);
    std::vector<int32_t> buf(64), paths((size_t)(n + 8) * 64, 0), plen(n + 8);
    int32_t len = 0, node = 0;
    for (int i = 0; i < n; ++i) {
        CHECK(cp_index_aligned(idx, i, buf.data(), 64, &len) == 0 && len == L[i]);
        CHECK(cp_index_path(idx, i, &paths[(size_t)i * 64], 64, &plen[i]) == 0);
        CHECK(cp_index_leaf(idx, i, &node) == 0 && node > 0 && node < nodes);
    }
    CHECK(cp_index_aligned(idx, 0, buf.data(), 0, &len) == -2 && len == L[0]);
    CHECK(cp_index_aligned(idx, n, buf.data(), 64, &len) == -2);
    for (int32_t v = 0; v < nodes; ++v) {
        int32_t parent, leaf, freq, nch;
        double at;
        CHECK(cp_index_node(idx, v, &parent, &leaf, &freq, &at, &nch, buf.data(), 64, &len) == 0);
        CHECK(cp_index_children(idx, v, buf.data(), 64, &len) == 0 && len == nch);
    }
    // insertion: a too small path buffer leaves the index untouched, the retry stores the context once
    const int32_t fresh[4] = {C[0], 31, 32, C[1] >= 0 && C[1] != C[0] ? C[1] : 33};
    int32_t aligned[4], path_len = 0;
    const int32_t before_nodes = cp_index_num_nodes(idx), before_ctx = cp_index_num_contexts(idx);
    CHECK(cp_index_insert(idx, fresh, 4, aligned, buf.data(), 0, &path_len) == -2 && path_len >= 1);
    CHECK(cp_index_num_nodes(idx) == before_nodes && cp_index_num_contexts(idx) == before_ctx);
    const int32_t bound = path_len;
    CHECK(cp_index_insert(idx, fresh, 4, aligned, buf.data(), bound, &path_len) == 0 && path_len <= bound);
    CHECK(cp_index_num_contexts(idx) == before_ctx + 1);
    CHECK(cp_index_search(idx, fresh, 4, buf.data(), 64, &len, &node) == 0);
    const int32_t twice[3] = {5, 5, 6};
    CHECK(cp_index_insert(idx, twice, 3, aligned, buf.data(), 64, &path_len) == -2);
    CHECK(cp_index_insert(idx, nullptr, 0, nullptr, buf.data(), 64, &path_len) == 0); // the empty context
    std::vector<int32_t> order(n);
    CHECK(cp_index_schedule(paths.data(), plen.data(), n, 64, order.data()) == 0);
    std::vector<int> seen(n, 0);
    for (int32_t o : order) {
        CHECK(o >= 0 && o < n);
        seen[o]++;
    }
    for (int s : seen) CHECK(s == 1);
    cp_index_free(idx);
    cp_index_free(nullptr);
    // the same batch with a distance matrix handed in
    std::vector<int32_t> rep(m);
    for (int i = n - 1; i >= 0; --i) rep[first_of[i]] = i;
    std::vector<float> dm((size_t)m * m);
    for (int a = 0; a < m; ++a)
        for (int b = 0; b < m; ++b) dm[(size_t)a * m + b] = (float)dist[(size_t)rep[a] * n + rep[b]];
    CHECK(cp_index_build(C.data(), L.data(), n, stride, 0.001, dm.data(), m, &idx) == 0);
    cp_index_free(idx);
    CHECK(cp_index_build(C.data(), L.data(), n, stride, 0.001, dm.data(), m + 1, &idx) != 0);
}

static void dedup()
{
    std::vector<std::string> blocks;
    for (int b = 0; b < 6; ++b) {
        std::string s;
        for (int l = 0; l < 30; ++l) {
            const int shared = (l % 3 == 0); // every third line is common to all blocks
            s += "line " + std::to_string(shared ? l : l * 100 + b) + " of the text\n";
        }
        if (b == 5) s += "no newline at the end";
        blocks.push_back(s);
    }
    CHECK(cp_dedup_hash((const uint8_t *)"a", 1) == 0xaf63dc4c8601ec8cULL); // FNV-1a 64 of "a"
    int64_t ends[64];
    int32_t cnt = 0;
    CHECK(cp_dedup_chunks((const uint8_t *)blocks[0].data(), (int64_t)blocks[0].size(), 4, ends, 64, &cnt) == 0);
    CHECK(cnt >= 1 && ends[cnt - 1] == (int64_t)blocks[0].size());
    CHECK(cp_dedup_chunks((const uint8_t *)blocks[0].data(), (int64_t)blocks[0].size(), 4, ends, 0, &cnt) == -2);
    cp_dedup *conv = nullptr;
    CHECK(cp_dedup_create(4, &conv) == 0 && conv);
    const int turns[3][3] = {{0, 1, 2}, {1, 3, 5}, {5, 4, 0}};
    for (int t = 0; t < 3; ++t) {
        std::string data;
        int64_t offsets[4];
        int32_t ids[3], ref[3];
        for (int i = 0; i < 3; ++i) {
            offsets[i] = (int64_t)data.size();
            ids[i] = turns[t][i];
            data += blocks[turns[t][i]];
        }
        offsets[3] = (int64_t)data.size();
        std::vector<cp_dedup_sub> subs(128);
        int64_t kept = 0;
        if (t == 1) { // a too small output leaves the conversation as it was
            CHECK(cp_dedup_turn(conv, ids, (const uint8_t *)data.data(), offsets, 3, ref, subs.data(), 1, &cnt, &kept) == -2);
        }
        CHECK(cp_dedup_turn(conv, ids, (const uint8_t *)data.data(), offsets, 3, ref, subs.data(), 128, &cnt, &kept) == 0);
        CHECK(kept >= 0 && kept <= (int64_t)data.size());
        for (int i = 0; i < cnt; ++i) CHECK(subs[i].begin >= 0 && subs[i].end <= (int64_t)data.size() && subs[i].begin <= subs[i].end);
        if (t > 0) CHECK(kept < (int64_t)data.size());
    }
    cp_dedup_free(conv);
    cp_dedup_free(nullptr);
}

int main()
{
    attention_and_cache_write();
    distances_index_and_schedule();
    dedup();
    puts("sanitized host run: ok");
    return 0;
}
