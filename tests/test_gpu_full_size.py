"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times.

The fp64 oracle cannot compute these in full within a test, so each case compares a seeded
sample of rows (all q heads of each sampled row): one random row per q block, the first and last
rows of every request, rows around random block seams and around split boundaries.  The needle
test covers what a sample of nearly flat softmax rows cannot see: a mis-gathered page.
"""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import error_stats
from test_gpu_parity import _check, _needle_case
from workloads import bf16_bits_to_f32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import gpu_harness
    return gpu_harness


def _sampled(H, w, rows, what, num_splits=0):
    got = H.gpu_attention(w, num_splits=num_splits)
    want = oracle.attention_of(w, rows=rows)
    st = _check(got[rows], want, f"{what}: sampled {len(rows)} of {w.total_extend} rows")
    assert np.isfinite(bf16_bits_to_f32(got)).all()
    return got


def test_config2_rag_fixed_sampled(H):
    w = W.config2_rag_fixed()
    assert w.num_pages == 5248 and w.total_extend == 18432
    rows = W.sample_rows(w, 2, q_block=128, edge=8, seams=4)
    _sampled(H, w, rows, "config2")


def test_config3_rag_zipf_sampled(H):
    w = W.config3_rag_zipf()
    print("config3 matched blocks", w.notes["matched_blocks"], "hit", w.notes["token_hit_ratio"])
    assert 0.05 < w.notes["token_hit_ratio"] < 0.5
    rows = W.sample_rows(w, 3, q_block=1024, edge=4, seams=2)
    _sampled(H, w, rows, "config3")


def test_config4_long_context_sampled_unsplit_and_split(H):
    w = W.config4_long_context()
    rows = W.sample_rows(w, 4, q_block=1024, edge=4, seams=3)
    a = _sampled(H, w, rows, "config4 unsplit", num_splits=1)
    # forced split-K over the 24576-token prefix; rows near the row-tile seams included above
    b = _sampled(H, w, rows, "config4 split=2", num_splits=2)
    d = np.abs(bf16_bits_to_f32(a).astype(np.float64) - bf16_bits_to_f32(b).astype(np.float64))
    assert d.max() <= 1e-3


def test_config5_128k_zero_reuse_and_reuse_sampled(H):
    wa = W.config5_128k(False)
    rows = W.sample_rows(wa, 5, q_block=2048, edge=4, seams=4)
    _sampled(H, wa, rows, "config5a zero reuse")
    del wa
    wb = W.config5_128k(True)
    rows = W.sample_rows(wb, 6, q_block=512, edge=4, seams=4)
    _sampled(H, wb, rows, "config5b 87.5% reuse")


def test_config5_reuse_run_equals_the_last_rows_of_the_zero_reuse_run(H):
    """Both 128k runs see the same token streams (the reuse run's pages hold the first 114688
    K/V rows of the zero-reuse run, its q / k_new / v_new are the last 16384 rows), so the two
    outputs must agree row for row: each is one bf16 rounding of nearly the same fp32 value, hence
    at most two bf16 steps apart."""
    wa = W.config5_128k(False)
    full = bf16_bits_to_f32(H.gpu_attention(wa)[114688:]).astype(np.float64)
    del wa
    wb = W.config5_128k(True)
    part = bf16_bits_to_f32(H.gpu_attention(wb)).astype(np.float64)
    assert part.shape == full.shape == (16384, 32, 128)
    step = np.maximum(np.abs(full), np.abs(part)) * 2.0 ** -7      # one bf16 step is at most 2^-7 of the value
    assert (np.abs(full - part) <= 2.0 * step + 1e-30).all()
    assert (full == part).mean() > 0.9


def _bench_workload(name):
    import bench
    return bench._workload(name)


@pytest.mark.parametrize("name,q_block", [("short_extend_probe", 64), ("rag_zipf_as_retrieved", 1024),
                                          ("rag_zipf_context_index", 1024), ("rag_fixed_shared_prefix", 128)])
def test_other_timed_extend_shapes_sampled(H, name, q_block):
    """Shapes that bench.py times beside the five configs, at the size timed: the short-extend
    probe (32 requests x 128 new tokens over 10240 cached, two q heads packed per workgroup) and
    the Zipf batch in the other two block orders (as retrieved; aligned and scheduled by the
    context index), and the fixed-reuse batch with all eight requests on one shared cached prefix."""
    w = _bench_workload(name)
    rows = W.sample_rows(w, 21, q_block=q_block, edge=4, seams=2)
    _sampled(H, w, rows, name)


def test_other_timed_decode_shapes(H):
    """decode_b32_p10k_e16: 16 new tokens per request (two blocks of 32 rows per KV head, four key
    chunks), every row checked.  decode_b1_p128k: one token over 131072 cached tokens, 256 key
    chunks merged."""
    w = _bench_workload("decode_b32_p10k_e16")
    assert w.total_extend == 512
    _check(H.gpu_attention(w), oracle.attention_of(w), "decode_b32_p10k_e16, all 512 rows")
    del w
    w = _bench_workload("decode_b1_p128k")
    import paper_2511_03475_amd as cp
    from gpu_harness import DeviceCase
    assert cp.cp_num_splits(DeviceCase(w).shape) == 256
    _check(H.gpu_attention(w), oracle.attention_of(w), "decode_b1_p128k")


def test_chunked_prefill_and_decode_workloads_sampled(H):
    """The other shapes bench.py times: one 2048-token chunk over 16k cached tokens, and the
    decode batch (32 requests x 10240 cached tokens, one new token each; decode-shaped kernel)."""
    w = W.make_uniform("chunked_prefill_b8_p16k_e2k", W.BASE_SEED + 10, 8, 32, 8, 16384, 2048)
    rows = W.sample_rows(w, 10, q_block=512, edge=2, seams=2)
    _sampled(H, w, rows, "chunked prefill")
    del w
    w = W.make_uniform("decode_b32_p10k", W.BASE_SEED + 7, 32, 32, 8, 10240, 1)
    got = H.gpu_attention(w)
    _check(got, oracle.attention_of(w), "decode batch, all 32 rows")


def test_needle_hits_every_page_at_128k(H):
    """P=114688, E=16384, 32/8 heads: each of the 8192 pages is the target of one query row."""
    P, E, PS = 114688, 16384, 16
    w, _, _, vals = _needle_case(P, E, 32, 8, 11, 0)
    rng = np.random.default_rng(11)
    n_pp, n_sp = P // PS, E // PS
    # suffix page s is targeted by its own last row (which sees the whole page); prefix pages
    # by the other rows
    suffix_rows = np.arange(n_sp) * PS + PS - 1
    other = np.setdiff1d(np.arange(E), suffix_rows)
    prefix_rows = rng.choice(other, size=n_pp, replace=False)
    rows = np.concatenate([prefix_rows, suffix_rows])
    targets = np.concatenate([np.arange(n_pp) * PS + rng.integers(0, PS, n_pp),
                              P + np.arange(n_sp) * PS + rng.integers(0, PS, n_sp)])
    assert (targets <= P + rows).all()
    nbits = int(P + E - 1).bit_length()
    keys = np.zeros((len(rows), 128), np.float32)
    for b in range(nbits):
        keys[:, b] = np.where((targets >> b) & 1, 8.0, -8.0)
    cq = np.float32(24.0 / (128.0 * w.softmax_scale))
    w.q[:] = 0
    w.q[rows] = W.f32_to_bf16_bits(keys * cq)[:, None, :]
    got = bf16_bits_to_f32(H.gpu_attention(w)).astype(np.float64)
    err = np.abs(got[rows] - vals[targets][:, None, :])
    bad = np.argwhere(err.max(axis=(1, 2)) > 1e-3)
    assert bad.size == 0, f"{bad.size} needle rows wrong, first: row {rows[bad[0, 0]]} target {targets[bad[0, 0]]}"
    # the oracle agrees on a few of them
    pick = np.sort(rng.choice(len(rows), size=6, replace=False))
    want = oracle.attention_of(w, rows=rows[pick].astype(np.int32))
    assert np.abs(want - vals[targets[pick]][:, None, :]).max() < 1e-6


@pytest.mark.parametrize("which", ["long_context_32k", "ctx128k_reuse"])
def test_full_size_closed_forms_on_every_row(H, which):
    """Two properties that hold at any size and need no sampled oracle, checked on EVERY row and
    head of the 32k workload (4 requests, 64/8 heads, P=24576, E=8192) and of the 128k reuse run
    (P=114688, E=16384): q = 0 makes all scores equal, so row i is the mean of the values of keys
    0 .. P+i of its KV head (a running mean, computed here in fp64 from the same bits); V = 1 makes
    every output 1."""
    w = W.config4_long_context() if which == "long_context_32k" else W.config5_128k(True)
    G = w.num_q_heads // w.num_kv_heads
    q_saved = w.q.copy()
    w.q[:] = 0
    got = bf16_bits_to_f32(H.gpu_attention(w)).astype(np.float64)            # [T, Hq, D]
    cu = w.cu_extend
    worst = 0.0
    for r in range(w.batch):
        P, E = int(w.prefix_lens[r]), int(w.extend_lens[r])
        pages = w.block_table[r, :P // 16]
        vp = bf16_bits_to_f32(w.kv_pages[pages, 1]).astype(np.float64)       # [pages, Hkv, 16, D]
        vp = vp.transpose(0, 2, 1, 3).reshape(P, w.num_kv_heads, 128)
        vn = bf16_bits_to_f32(w.v_new[cu[r]:cu[r] + E]).astype(np.float64)
        run = vp.sum(axis=0)[None] + np.cumsum(vn, axis=0)                   # sums over keys 0 .. P+i
        mean = run / (P + 1 + np.arange(E))[:, None, None]                   # [E, Hkv, D]
        want = np.repeat(mean, G, axis=1)                                    # q head h uses KV head h // G
        err = np.abs(got[cu[r]:cu[r] + E] - want)
        worst = max(worst, float(err.max()))
        # the means are ~N(0, 1/n): bf16 rounding of the output dominates the error
        assert err.max() <= 2.0 ** -8 * np.abs(want).max() + 1e-6, (r, err.max())
    print("running mean: worst abs error", worst)
    w.q[:] = q_saved
    w.v_new[:] = 0x3F80
    w.kv_pages[:, 1] = 0x3F80
    ones = bf16_bits_to_f32(H.gpu_attention(w))
    assert (ones == 1.0).all()
