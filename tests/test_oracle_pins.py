"""Pins of the fp64 CPU oracle against facts that do not come from the oracle itself.

The paper prints no worked numeric example for prefill attention over a prefix cache
(Section 1 and Section 2.1 describe it only as engine behaviour), so the oracle is pinned
by closed forms, invariants, brute force on tiny inputs and a library routine
(torch scaled_dot_product_attention in fp64) on dense gathers.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from helpers import case_from_floats, dense_kv
from workloads import bf16_bits_to_f32, f32_to_bf16_bits, make_uniform

TOL = 1e-12


def _rand_case(seed, B, Hq, Hkv, P, E, **kw):
    return make_uniform("t", seed, B, Hq, Hkv, P, E, **kw)


# ---------------------------------------------------------------- closed forms
def test_two_keys_closed_form():
    """Scores 0 and 1 (scale 1): weights are 1/(1+e) and e/(1+e)."""
    D, PS = 4, 2
    q = np.zeros((1, 1, D)); q[0, 0, 0] = 1.0
    pool = np.zeros((1, 2, 1, PS, D))
    pool[0, 0, 0, 0, :] = [0, 3, 0, 0]          # prefix key: score 0
    pool[0, 1, 0, 0, :] = [2, -1, 0.5, 8]       # prefix value
    k_new = np.zeros((1, 1, D)); k_new[0, 0, 0] = 1.0   # own key: score 1
    v_new = np.array([[[4.0, 1.0, -0.25, 0.0]]])
    w = case_from_floats(q, k_new, v_new, pool, [[0]], [1], [1], scale=1.0)
    out = oracle.attention_of(w)
    e = math.e
    want = (np.array([2, -1, 0.5, 8]) + e * np.array([4.0, 1.0, -0.25, 0.0])) / (1 + e)
    np.testing.assert_allclose(out[0, 0], want, rtol=0, atol=1e-15)


def test_uniform_keys_give_running_mean_of_values():
    w = _rand_case(11, 2, 4, 2, [37, 0], [19, 23])
    w.k_new[:] = w.k_new[0, 0]                  # every key identical
    w.kv_pages[:, 0] = w.k_new[0, 0]
    out = oracle.attention_of(w)
    for r in range(w.batch):
        _, V = dense_kv(w, r)
        P, E, cu = int(w.prefix_lens[r]), int(w.extend_lens[r]), int(w.cu_extend[r])
        csum = np.cumsum(V, axis=0)
        for i in range(E):
            mean = csum[P + i] / (P + i + 1)    # [Hkv, D]
            for h in range(w.num_q_heads):
                np.testing.assert_allclose(out[cu + i, h], mean[h // 2], rtol=0, atol=TOL)


def test_zero_query_gives_running_mean_of_values():
    w = _rand_case(12, 1, 2, 1, 21, 9)
    w.q[:] = 0
    out = oracle.attention_of(w)
    _, V = dense_kv(w, 0)
    for i in range(9):
        np.testing.assert_allclose(out[i, 1], V[:21 + i + 1, 0].mean(0), rtol=0, atol=TOL)


def test_value_all_ones_gives_ones():
    w = _rand_case(13, 2, 4, 2, [16, 5], [8, 11])
    one = f32_to_bf16_bits(np.float32(1.0))
    w.v_new[:] = one
    w.kv_pages[:, 1] = one
    out = oracle.attention_of(w)
    np.testing.assert_allclose(out, 1.0, rtol=0, atol=TOL)


# ---------------------------------------------------------------- brute force, tiny
def _brute(w):
    """exp / sum written out with Python loops, no max subtraction."""
    out = np.zeros((w.total_extend, w.num_q_heads, w.head_dim))
    G = w.num_q_heads // w.num_kv_heads
    qf = bf16_bits_to_f32(w.q).astype(np.float64)
    for r in range(w.batch):
        K, V = dense_kv(w, r)
        P, E, cu = int(w.prefix_lens[r]), int(w.extend_lens[r]), int(w.cu_extend[r])
        for i in range(E):
            for h in range(w.num_q_heads):
                g = h // G
                num = np.zeros(w.head_dim)
                den = 0.0
                for j in range(P + i + 1):
                    s = 0.0
                    for d in range(w.head_dim):
                        s += qf[cu + i, h, d] * K[j, g, d]
                    e = math.exp(w.softmax_scale * s)
                    den += e
                    num += e * V[j, g]
                out[cu + i, h] = num / den
    return out


@pytest.mark.parametrize("D,PS", [(4, 2), (128, 16)])
def test_brute_force_tiny(D, PS):
    rng = np.random.default_rng(5)
    B, Hq, Hkv = 2, 4, 2
    P, E = [3, 0], [4, 5]
    T = sum(E)
    npages = 6
    w = case_from_floats(rng.standard_normal((T, Hq, D)), rng.standard_normal((T, Hkv, D)),
                         rng.standard_normal((T, Hkv, D)),
                         rng.standard_normal((npages, 2, Hkv, PS, D)),
                         [[4, 1, 5, 0], [2, 3, 0, 0]] if PS == 2 else [[4], [2]], P, E)
    np.testing.assert_allclose(oracle.attention_of(w), _brute(w), rtol=0, atol=1e-13)


# ---------------------------------------------------------------- library routine
def _sdpa(w):
    out = np.zeros((w.total_extend, w.num_q_heads, w.head_dim))
    G = w.num_q_heads // w.num_kv_heads
    for r in range(w.batch):
        K, V = dense_kv(w, r)
        P, E, cu = int(w.prefix_lens[r]), int(w.extend_lens[r]), int(w.cu_extend[r])
        if E == 0:
            continue
        q = torch.from_numpy(bf16_bits_to_f32(w.q[cu:cu + E]).astype(np.float64)).permute(1, 0, 2)
        k = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, dim=0)
        v = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, dim=0)
        mask = torch.arange(P + E)[None, :] <= (P + torch.arange(E))[:, None]
        o = torch.nn.functional.scaled_dot_product_attention(
            q[None], k[None], v[None], attn_mask=mask, scale=w.softmax_scale)[0]
        out[cu:cu + E] = o.permute(1, 0, 2).numpy()
    return out


def test_prefix_zero_is_plain_causal_attention():
    w = _rand_case(21, 1, 4, 2, 0, 70)
    q = torch.from_numpy(bf16_bits_to_f32(w.q).astype(np.float64)).permute(1, 0, 2)[None]
    k = torch.from_numpy(bf16_bits_to_f32(w.k_new).astype(np.float64)).permute(1, 0, 2)
    v = torch.from_numpy(bf16_bits_to_f32(w.v_new).astype(np.float64)).permute(1, 0, 2)
    k = k.repeat_interleave(2, dim=0)[None]
    v = v.repeat_interleave(2, dim=0)[None]
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)[0]
    np.testing.assert_allclose(oracle.attention_of(w), want.permute(1, 0, 2).numpy(),
                               rtol=0, atol=TOL)


def test_paged_extend_matches_sdpa_on_dense_gather():
    w = _rand_case(22, 3, 8, 2, [45, 0, 130], [33, 17, 1], num_pages=40)
    np.testing.assert_allclose(oracle.attention_of(w), _sdpa(w), rtol=0, atol=TOL)


# ---------------------------------------------------------------- seam, paging
@pytest.mark.parametrize("P", [1, 15, 16, 17, 40, 63])
def test_one_pass_equals_cache_then_extend(P):
    N = 64
    full = _rand_case(31, 1, 4, 2, 0, N, num_pages=8)
    out_full = oracle.attention_of(full)
    pool = oracle.write_kv(full.k_new[:P], full.v_new[:P], full.kv_pages, full.block_table,
                           np.array([0], np.int32), np.array([P], np.int32))
    out_ext = oracle.extend_attention(full.q[P:], full.k_new[P:], full.v_new[P:], pool,
                                      full.block_table, np.array([P], np.int32),
                                      np.array([N - P], np.int32), full.softmax_scale)
    np.testing.assert_allclose(out_ext, out_full[P:], rtol=0, atol=TOL)


def test_page_permutation_invariance():
    w = _rand_case(32, 2, 4, 2, [50, 33], [10, 20], num_pages=16)
    base = oracle.attention_of(w)
    perm = np.random.default_rng(1).permutation(w.num_pages)   # new physical index of page p
    pool2 = np.empty_like(w.kv_pages)
    pool2[perm] = w.kv_pages
    table2 = np.where(w.block_table >= 0, perm[np.maximum(w.block_table, 0)], -1)
    out = oracle.extend_attention(w.q, w.k_new, w.v_new, pool2, table2, w.prefix_lens,
                                  w.extend_lens, w.softmax_scale)
    np.testing.assert_array_equal(out, base)


def test_needle_selects_the_right_token_of_every_page():
    """A query that scores one key far above the rest must return that key's value row."""
    B, Hq, Hkv, D, PS = 1, 2, 1, 128, 16
    P, E = 96, 32
    w = _rand_case(33, B, Hq, Hkv, P, E, num_pages=16)
    N = P + E
    # value row of logical token t encodes t in bf16-exact integers
    def code(t):
        v = np.zeros(D, np.float32); v[0] = t % 128; v[1] = t // 128; v[2] = 1.0
        return f32_to_bf16_bits(v)
    # key of token t: one-hot-ish +-8 pattern from the bits of t (exact in bf16)
    def keyvec(t):
        k = np.zeros(D, np.float32)
        for b in range(8):
            k[b] = 8.0 if (t >> b) & 1 else -8.0
        return k
    for t in range(N):
        kb, vb = f32_to_bf16_bits(keyvec(t)), code(t)
        if t < P:
            pg, sl = w.block_table[0, t // PS], t % PS
            w.kv_pages[pg, 0, 0, sl], w.kv_pages[pg, 1, 0, sl] = kb, vb
        else:
            w.k_new[t - P, 0], w.v_new[t - P, 0] = kb, vb
    rng = np.random.default_rng(2)
    targets = [int(rng.integers(0, P + i + 1)) for i in range(E)]
    targets[0], targets[-1] = 0, N - 1
    for i, t in enumerate(targets):
        w.q[i, :] = f32_to_bf16_bits(keyvec(t) * 2.0)
    out = oracle.attention_of(w)
    # matching key scores 8*8*16*scale = 90.5; any other key differs in >= 1 bit: <= 67.9
    for i, t in enumerate(targets):
        want = bf16_bits_to_f32(code(t)).astype(np.float64)
        np.testing.assert_allclose(out[i, 0], want, rtol=0, atol=1e-6)
        np.testing.assert_allclose(out[i, 1], want, rtol=0, atol=1e-6)


# ---------------------------------------------------------------- invariances
def test_key_shift_invariance_with_large_scores():
    w = _rand_case(41, 1, 2, 1, 30, 12)
    # add a constant vector c to every key: scores of a row all move by scale * q.c
    c = np.zeros(128, np.float32); c[:4] = 64.0
    def shift(bits):
        f = bf16_bits_to_f32(bits)
        f[..., :4] = 0.0                 # make the sum exact in bf16: only c lives in dims 0..3
        return f
    k0 = shift(w.k_new); p0 = shift(w.kv_pages[:, 0])
    w.k_new = f32_to_bf16_bits(k0); w.kv_pages[:, 0] = f32_to_bf16_bits(p0)
    base = oracle.attention_of(w)
    w.k_new = f32_to_bf16_bits(k0 + c); w.kv_pages[:, 0] = f32_to_bf16_bits(p0 + c)
    shifted = oracle.attention_of(w)
    qf = bf16_bits_to_f32(w.q).astype(np.float64)
    assert np.abs(qf[..., :4].sum(-1) * 64.0 * w.softmax_scale).max() > 20.0
    np.testing.assert_allclose(shifted, base, rtol=0, atol=1e-9)


def test_linearity_in_values():
    w = _rand_case(42, 2, 4, 2, [20, 3], [6, 9])
    rng = np.random.default_rng(3)
    def small_ints(shape):
        return rng.integers(-8, 9, size=shape).astype(np.float32)
    v1n, v2n = small_ints(w.v_new.shape), small_ints(w.v_new.shape)
    v1p, v2p = small_ints(w.kv_pages[:, 1].shape), small_ints(w.kv_pages[:, 1].shape)
    def run(vn, vp):
        w.v_new = f32_to_bf16_bits(vn); w.kv_pages[:, 1] = f32_to_bf16_bits(vp)
        return oracle.attention_of(w)
    o1, o2 = run(v1n, v1p), run(v2n, v2p)
    o3 = run(2 * v1n - 3 * v2n, 2 * v1p - 3 * v2p)     # exact in bf16 (|.| <= 40)
    np.testing.assert_allclose(o3, 2 * o1 - 3 * o2, rtol=0, atol=1e-11)


def test_causality_future_tokens_do_not_matter():
    w = _rand_case(43, 1, 2, 1, 10, 24)
    base = oracle.attention_of(w)
    i = 9
    w.k_new[i + 1:] ^= 0x0101
    w.v_new[i + 1:] ^= 0x0301
    out = oracle.attention_of(w)
    np.testing.assert_array_equal(out[:i + 1], base[:i + 1])
    assert np.abs(out[i + 1:] - base[i + 1:]).max() > 1e-3


def test_gqa_head_mapping():
    w = _rand_case(44, 1, 6, 3, 12, 7)             # G = 2: heads (0,1)->kv0, (2,3)->kv1, (4,5)->kv2
    w.q[:, 1] = w.q[:, 0]; w.q[:, 3] = w.q[:, 0]; w.q[:, 5] = w.q[:, 0]
    w.q[:, 2] = w.q[:, 0]; w.q[:, 4] = w.q[:, 0]
    out = oracle.attention_of(w)
    np.testing.assert_array_equal(out[:, 0], out[:, 1])
    np.testing.assert_array_equal(out[:, 2], out[:, 3])
    assert np.abs(out[:, 0] - out[:, 2]).max() > 1e-3
    # swapping KV heads 0 and 2 swaps the outputs of their groups
    w.k_new[:, [0, 2]] = w.k_new[:, [2, 0]]; w.v_new[:, [0, 2]] = w.v_new[:, [2, 0]]
    w.kv_pages[:, :, [0, 2]] = w.kv_pages[:, :, [2, 0]]
    out2 = oracle.attention_of(w)
    np.testing.assert_array_equal(out2[:, 0], out[:, 4])
    np.testing.assert_array_equal(out2[:, 4], out[:, 0])
    np.testing.assert_array_equal(out2[:, 2], out[:, 2])


def test_split_key_ranges_merge_to_the_whole():
    """Log-sum-exp algebra: attention over S1 u S2 is the lse-weighted mix of the parts."""
    w = _rand_case(45, 2, 4, 2, [40, 7], [13, 21])
    full, lse = oracle.attention_of(w, return_lse=True)
    cuts = [0, 9, 33, 10 ** 6]
    parts = [oracle.attention_of(w, key_lo=a, key_hi=b, return_lse=True)
             for a, b in zip(cuts[:-1], cuts[1:])]
    lses = np.stack([p[1] for p in parts])                 # [S, T, Hq], -inf where empty
    m = lses.max(0)
    wts = np.exp(lses - m)
    mix = sum(wts[s][..., None] * parts[s][0] for s in range(len(parts))) / wts.sum(0)[..., None]
    np.testing.assert_allclose(mix, full, rtol=0, atol=TOL)
    np.testing.assert_allclose(m + np.log(wts.sum(0)), lse, rtol=0, atol=TOL)


# ---------------------------------------------------------------- cache write
def test_write_kv_places_rows_and_leaves_the_rest():
    w = _rand_case(51, 3, 4, 2, [5, 32, 0], [20, 1, 33], num_pages=12)
    sentinel = np.uint16(0x7FC1)
    pool0 = np.full_like(w.kv_pages, sentinel)
    got = oracle.write_kv(w.k_new, w.v_new, pool0, w.block_table, w.prefix_lens, w.extend_lens)
    want = pool0.copy()
    cu = w.cu_extend
    for r in range(w.batch):
        for j in range(int(w.extend_lens[r])):
            t = int(w.prefix_lens[r]) + j
            pg, sl = w.block_table[r, t // 16], t % 16
            want[pg, 0, :, sl, :] = w.k_new[cu[r] + j]
            want[pg, 1, :, sl, :] = w.v_new[cu[r] + j]
    np.testing.assert_array_equal(got, want)
    assert (got == sentinel).sum() == got.size - 2 * w.total_extend * w.num_kv_heads * 128
    np.testing.assert_array_equal(pool0, np.full_like(pool0, sentinel))   # input untouched


def test_empty_and_degenerate_requests():
    w = _rand_case(52, 3, 2, 1, [16, 0, 5], [0, 1, 0])
    out = oracle.attention_of(w)
    assert out.shape == (1, 2, 128)
    v = bf16_bits_to_f32(w.v_new[0, 0]).astype(np.float64)
    np.testing.assert_allclose(out[0, 0], v, rtol=0, atol=TOL)   # single visible key: itself
