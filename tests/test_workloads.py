"""Host-side checks of the synthetic workload generators (structure only, no attention)."""
import numpy as np

import workloads as W


def _check_tables(w):
    ps = w.page_size
    for r in range(w.batch):
        need = (int(w.prefix_lens[r]) + int(w.extend_lens[r]) + ps - 1) // ps
        row = w.block_table[r]
        assert need <= w.max_pages_per_req
        assert (row[:need] >= 0).all() and (row[:need] < w.num_pages).all()
        assert len(set(row[:need].tolist())) == need
    assert w.q.shape == (w.total_extend, w.num_q_heads, 128)
    assert w.k_new.shape == w.v_new.shape == (w.total_extend, w.num_kv_heads, 128)
    assert w.kv_pages.shape == (w.num_pages, 2, w.num_kv_heads, 16, 128)


def test_bf16_rounding_is_nearest_even_and_round_trips():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.140625], np.float32)
    b = W.f32_to_bf16_bits(x)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: even mantissa wins; 1 + 3*2^-8 ties up
    np.testing.assert_array_equal(W.bf16_bits_to_f32(b),
                                  np.array([1.0, 1.0, 1.015625, -2.5, 0.0, 3.140625], np.float32))
    again = W.f32_to_bf16_bits(W.bf16_bits_to_f32(b))
    np.testing.assert_array_equal(again, b)


def test_config1_shape_and_determinism():
    a, b = W.config1_tiny(), W.config1_tiny()
    _check_tables(a)
    assert (a.batch, a.num_q_heads, a.num_kv_heads, a.num_pages) == (1, 8, 2, 64)
    assert a.prefix_lens.tolist() == [512] and a.extend_lens.tolist() == [128]
    assert a.pairs_per_head() == 73792 and abs(a.flops() - 3.0225e8) < 1e5
    np.testing.assert_array_equal(a.q, b.q)
    np.testing.assert_array_equal(a.block_table, b.block_table)
    f = W.bf16_bits_to_f32(a.q).astype(np.float64)
    assert abs(f.mean()) < 0.02 and abs(f.std() - 1.0) < 0.02


def test_config2_small_page_regions():
    w = W.config2_rag_fixed(batch=2, block=64, Hq=4, Hkv=2, query=16, cached_region_pages=64)
    _check_tables(w)
    pp = 6 * 64 // 16
    assert (w.block_table[:, :pp] < 64).all() and (w.block_table[:, pp:] >= 64).all()
    assert w.prefix_lens.tolist() == [384, 384] and w.extend_lens.tolist() == [144, 144]
    # destination pages of different requests never collide
    dest = w.block_table[:, pp:].ravel()
    assert len(set(dest.tolist())) == dest.size


def test_config3_small_zipf_alignment_and_aliasing():
    w = W.config3_rag_zipf(batch=16, block=32, topk=6, pool_ids=40, query=16, Hq=4, Hkv=2)
    m = w.notes["matched_blocks"]
    assert m[0] == 0 and max(m) >= 1
    bp = 32 // 16
    for r in range(w.batch):
        assert w.prefix_lens[r] == 32 * m[r] and w.extend_lens[r] == 32 * (6 - m[r]) + 16
        if m[r]:
            # the cached prefix pages are exactly some earlier request's leading pages
            assert any((w.block_table[e, :m[r] * bp] == w.block_table[r, :m[r] * bp]).all()
                       for e in range(r))
        # destination pages (tokens >= P_r) are private to the request
        mine = set(w.block_table[r, m[r] * bp:].tolist())
        for e in range(w.batch):
            if e != r:
                assert not (mine & set(w.block_table[e, m[e] * bp:].tolist()))
    assert 0.0 < w.notes["token_hit_ratio"] < 1.0


def test_sample_rows_cover_edges_and_every_block():
    w = W.make_uniform("s", 3, 2, 2, 1, [64, 0], [700, 130])
    rows = W.sample_rows(w, 9, q_block=128, edge=4, seams=3, extra_boundaries=[300])
    assert rows.dtype == np.int32 and (np.diff(rows) > 0).all()
    s = set(rows.tolist())
    assert {0, 1, 2, 3, 696, 697, 698, 699, 299, 300, 301, 700, 829}.issubset(s)
    for blk in range(6):
        assert any(blk * 128 <= x < min((blk + 1) * 128, 700) for x in s)


def test_rag_batch_from_blocks_prefix_matching_and_order():
    ctx = [[5, 6, 7], [5, 6, 9], [1], [5, 2]]
    w = W.rag_batch_from_blocks("t", 77, ctx, block=32, query=16, Hq=4, Hkv=2)
    assert w.notes["matched_blocks"] == [0, 2, 0, 1]
    assert list(w.prefix_lens) == [0, 64, 0, 32] and list(w.extend_lens) == [112, 48, 48, 48]
    # prefix pages alias the donor's pages; everything else is distinct
    assert list(w.block_table[1, :4]) == list(w.block_table[0, :4])
    assert list(w.block_table[3, :2]) == list(w.block_table[0, :2])
    used = [int(p) for r in range(4) for p in w.block_table[r] if p >= 0]
    assert len(set(used)) == w.num_pages and max(used) == w.num_pages - 1
    # execution order: request r of the batch is ctx[order[r]]
    w2 = W.rag_batch_from_blocks("t", 77, ctx, block=32, query=16, Hq=4, Hkv=2, order=[3, 1, 0, 2])
    assert w2.notes["matched_blocks"] == [0, 1, 2, 0]
    assert list(w2.prefix_lens) == [0, 32, 64, 0]


def test_config3_is_the_frequency_sorted_special_case():
    picks = W.rag_zipf_picks(batch=6, topk=4, pool_ids=12)
    assert len(picks) == 6 and all(len(set(p)) == 4 for p in picks)
    assert W.rag_zipf_picks(batch=6, topk=4, pool_ids=12) == picks, "seeded"


def test_config5_runs_share_their_token_streams():
    """The reuse run is the zero-reuse run with its first rows moved into the cache: same q / k / v
    bits for the last rows, same block table, pages filled with the first rows' K/V."""
    total, cached = 4096 + 160, 4096
    a, b = W.config5_128k(False, total=total, cached=cached), W.config5_128k(True, total=total, cached=cached)
    _check_tables(a)
    _check_tables(b)
    assert a.prefix_lens.tolist() == [0] and b.prefix_lens.tolist() == [cached]
    np.testing.assert_array_equal(b.q, a.q[cached:])
    np.testing.assert_array_equal(b.k_new, a.k_new[cached:])
    np.testing.assert_array_equal(b.v_new, a.v_new[cached:])
    np.testing.assert_array_equal(a.block_table, b.block_table)
    for tok in (0, 15, 16, 2047, cached - 1):
        page, slot = b.block_table[0, tok // 16], tok % 16
        np.testing.assert_array_equal(b.kv_pages[page, 0, :, slot, :], a.k_new[tok])
        np.testing.assert_array_equal(b.kv_pages[page, 1, :, slot, :], a.v_new[tok])
    # rows drawn on their own equal the same rows of the whole array
    import workloads.generate as G
    whole = G.normal_bf16(np.random.default_rng(5), (3000, 7, 128), chunk_elems=1 << 16)
    part = G.normal_bf16_rows(np.random.default_rng(5), (3000, 7, 128), 1234, 2999, chunk_elems=1 << 16)
    np.testing.assert_array_equal(part, whole[1234:2999])
