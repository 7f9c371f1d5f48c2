// Driver for the sanitizer build of the HOST side of the C ABI (argument checks and launch
// planning in cp_extend.hip; the device code is compiled without instrumentation).  No kernel is
// launched: every call here returns from its host-side checks, or is a planning query.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "cp_extend.h"

#define CHECK(c)                                                                  \
    do {                                                                          \
        if (!(c)) {                                                               \
            fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #c); \
            exit(1);                                                              \
        }                                                                         \
    } while (0)

static cp_shape shape_of(const std::vector<int32_t> &P, const std::vector<int32_t> &E, int Hq, int Hkv, int splits)
{
    cp_shape s{};
    s.batch = (int32_t)P.size();
    s.num_q_heads = Hq;
    s.num_kv_heads = Hkv;
    s.head_dim = 128;
    s.page_size = 16;
    s.num_pages = 1 << 20;
    int32_t width = 1;
    int64_t total = 0;
    for (size_t r = 0; r < P.size(); ++r) {
        const int32_t need = (P[r] + E[r] + 15) / 16;
        width = need > width ? need : width;
        total += E[r];
    }
    s.max_pages_per_req = width;
    s.total_extend = (int32_t)total;
    s.softmax_scale = 0.0883883f;
    s.num_splits = splits;
    s.h_prefix_lens = P.data();
    s.h_extend_lens = E.data();
    return s;
}

int main()
{
    void *const ptr = (void *)(uintptr_t)4096; // never dereferenced on the host
    const int32_t *const iptr = (const int32_t *)ptr;
    {
        const std::vector<int32_t> P(4, 24576), E(4, 8192);
        cp_shape s = shape_of(P, E, 64, 8, 0);
        CHECK(cp_num_splits(&s) == 1 && cp_workspace_bytes(&s) == 0 && cp_plan_kind(&s) == CP_PLAN_ROW_TILED);
        s.num_splits = 2;
        CHECK(cp_num_splits(&s) == 2 && cp_plan_kind(&s) == CP_PLAN_ROW_TILED_SPLIT);
        CHECK(cp_workspace_bytes(&s) == (size_t)2 * 4 * 8192 * 64 * 130 * 4);
        CHECK(cp_extend_attention(ptr, ptr, ptr, ptr, iptr, iptr, iptr, ptr, nullptr, &s, nullptr, 0) == CP_ERR_WORKSPACE);
        CHECK(cp_extend_attention_noalloc(ptr, ptr, ptr, ptr, iptr, iptr, iptr, ptr, nullptr, &s) == CP_ERR_WORKSPACE);
    }
    {
        std::vector<int32_t> P(200), E(200);
        for (int r = 0; r < 200; ++r) {
            P[r] = (r * 37) % 5000;
            E[r] = r % 7 == 0 ? 0 : 1 + (r * 13) % 3;
        }
        cp_shape s = shape_of(P, E, 32, 8, 0);
        CHECK(cp_plan_kind(&s) == CP_PLAN_DECODE && cp_num_splits(&s) % 4 == 0 && cp_workspace_bytes(&s) > 0);
        CHECK(cp_extend_attention(nullptr, ptr, ptr, ptr, iptr, iptr, iptr, ptr, nullptr, &s, nullptr, 0) == CP_ERR_NULL);
        CHECK(cp_extend_attention((void *)(uintptr_t)4104, ptr, ptr, ptr, iptr, iptr, iptr, ptr, nullptr, &s, nullptr, 0) == CP_ERR_ALIGN);
        CHECK(cp_write_kv(ptr, ptr, ptr, (const int32_t *)(uintptr_t)4098, iptr, iptr, nullptr, &s) == CP_ERR_ALIGN);
        CHECK(cp_check_tables(nullptr, iptr, iptr, nullptr, &s, nullptr) == CP_ERR_NULL);
        s.total_extend += 1;
        CHECK(cp_num_splits(&s) == 0 && cp_plan_kind(&s) == CP_PLAN_INVALID);
        CHECK(cp_write_kv(ptr, ptr, ptr, iptr, iptr, iptr, nullptr, &s) == CP_ERR_SHAPE);
    }
    {
        const std::vector<int32_t> P{0, 16}, E{0, 0}; // nothing to do: returns before any pointer is looked at
        cp_shape s = shape_of(P, E, 4, 2, 0);
        CHECK(cp_extend_attention(nullptr, nullptr, nullptr, nullptr, iptr, iptr, iptr, nullptr, nullptr, &s, nullptr, 0) == CP_OK);
        CHECK(cp_write_kv(nullptr, nullptr, nullptr, iptr, iptr, iptr, nullptr, &s) == CP_OK);
    }
    CHECK(cp_num_splits(nullptr) == 0 && cp_workspace_bytes(nullptr) == 0);
    for (int code = 0; code >= -8; --code) CHECK(cp_status_string(code) != nullptr);
    CHECK(cp_noalloc_scratch_bytes() == (size_t)64 << 20);
    puts("sanitized C-ABI host run: ok");
    return 0;
}
