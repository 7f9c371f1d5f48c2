"""GPU parity: the HIP path against the fp64 oracle on the same seeded inputs.

Tolerances (bf16 inputs, fp32 accumulation, bf16 output): max-abs <= 2e-2 and mean-abs <= 2e-3
over all compared elements, plus an error relative to the oracle's output RMS <= 2e-2, which
stays meaningful at long context where the outputs themselves are ~1e-2.
"""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import error_stats
from workloads import bf16_bits_to_f32, f32_to_bf16_bits

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS, REL_RMS = 2e-2, 2e-3, 2e-2


def _check(got_bits, want, what=""):
    got = bf16_bits_to_f32(got_bits).astype(np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    st = error_stats(got, want)
    print(f"[parity] {what}: {st}", flush=True)
    assert st["max_abs"] <= MAX_ABS, (what, st)
    assert st["mean_abs"] <= MEAN_ABS, (what, st)
    assert st["rel_rms"] <= REL_RMS, (what, st)
    return st


@pytest.fixture(scope="module")
def H():
    import gpu_harness
    return gpu_harness


def test_config1_tiny_full(H):
    w = W.config1_tiny()
    _check(H.gpu_attention(w), oracle.attention_of(w), "config1")


@pytest.mark.parametrize("P,E", [
    ([45, 0, 300], [33, 257, 130]),      # ragged: partial pages, partial q tiles, P = 0
    ([1, 63, 64, 65], [1, 127, 128, 129]),
    ([16, 0, 5], [0, 1, 0]),             # empty requests
    ([700], [391]),
])
def test_small_ragged_batches(H, P, E):
    w = W.make_uniform("ragged", 101, len(P), 8, 2, P, E)
    _check(H.gpu_attention(w), oracle.attention_of(w), f"ragged P={P} E={E}")


@pytest.mark.parametrize("G,Hkv", [(1, 2), (2, 3), (8, 1)])
def test_gqa_group_sizes(H, G, Hkv):
    w = W.make_uniform("gqa", 102, 2, G * Hkv, Hkv, [130, 17], [70, 200])
    _check(H.gpu_attention(w), oracle.attention_of(w), f"G={G} Hkv={Hkv}")


@pytest.mark.parametrize("G,Hkv,E", [
    (4, 2, [1, 17, 32]), (4, 2, [33, 64, 100]), (4, 2, [128, 129, 5]),
    (8, 1, [1, 31, 40]), (8, 1, [64, 65, 256]), (6, 1, [20, 70, 130]), (2, 3, [127, 3, 257]),
])
def test_short_extends_pack_several_heads_per_workgroup(H, G, Hkv, E):
    """Short extends share one workgroup's K/V tiles between q heads of a KV head."""
    w = W.make_uniform("pack", 111, len(E), G * Hkv, Hkv, [300, 0, 77], E)
    want = oracle.attention_of(w)
    _check(H.gpu_attention(w), want, f"pack G={G} E={E}")
    _check(H.gpu_attention(w, num_splits=3), want, f"pack split G={G} E={E}")


@pytest.mark.parametrize("ns", [2, 3, 7, 64])
def test_forced_split_k_matches_and_is_deterministic(H, ns):
    w = W.make_uniform("split", 103, 2, 4, 2, [1000, 37], [300, 150])
    want = oracle.attention_of(w)
    a = H.gpu_attention(w, num_splits=ns)
    _check(a, want, f"split={ns}")
    b = H.gpu_attention(w, num_splits=ns)
    np.testing.assert_array_equal(a, b)
    # splitting only regroups fp32 partial sums
    one = bf16_bits_to_f32(H.gpu_attention(w, num_splits=1)).astype(np.float64)
    assert np.abs(bf16_bits_to_f32(a).astype(np.float64) - one).max() <= 1e-2


def test_auto_split_on_short_extend(H):
    import paper_2511_03475_amd as cp
    w = W.make_uniform("short", 104, 2, 8, 2, 4096, 64)
    case = H.DeviceCase(w)
    assert cp.cp_num_splits(case.shape) > 1 and case.ws_bytes > 0
    case.attention()
    _check(case.out_bits(), oracle.attention_of(w), "auto split short extend")


def test_write_kv_bit_exact_and_sentinel(H):
    w = W.make_uniform("wkv", 105, 3, 4, 2, [5, 32, 0], [20, 1, 333], num_pages=40)
    w.kv_pages[:] = 0x7FC1
    case = H.DeviceCase(w)
    case.write_kv()
    want = oracle.write_kv(w.k_new, w.v_new, w.kv_pages, w.block_table, w.prefix_lens, w.extend_lens)
    np.testing.assert_array_equal(case.pool_bits(), want)


def test_write_then_extend_equals_one_pass(H):
    N, Hq, Hkv = 600, 8, 2
    full = W.make_uniform("seam", 106, 1, Hq, Hkv, 0, N, num_pages=40)
    want = oracle.attention_of(full)
    one_pass = H.gpu_attention(full)
    _check(one_pass, want, "one pass")
    for P in (1, 17, 64, 333, 599):
        # cache the first P tokens with the GPU cache write, then extend with the rest
        import copy
        head = copy.copy(full)
        head.prefix_lens = np.array([0], np.int32); head.extend_lens = np.array([P], np.int32)
        head.q, head.k_new, head.v_new = full.q[:P], full.k_new[:P], full.v_new[:P]
        hc = H.DeviceCase(head)
        hc.write_kv()
        tail = copy.copy(full)
        tail.prefix_lens = np.array([P], np.int32); tail.extend_lens = np.array([N - P], np.int32)
        tail.q, tail.k_new, tail.v_new = full.q[P:], full.k_new[P:], full.v_new[P:]
        tail.kv_pages = hc.pool_bits()
        got = H.gpu_attention(tail)
        _check(got, want[P:], f"cache {P} then extend {N - P}")
        d = np.abs(bf16_bits_to_f32(got).astype(np.float64) -
                   bf16_bits_to_f32(one_pass[P:]).astype(np.float64))
        assert d.max() <= 2e-2      # two bf16 roundings of values up to ~4


def test_page_permutation_is_bitwise_invariant(H):
    w = W.make_uniform("perm", 107, 2, 8, 2, [500, 130], [100, 200], num_pages=80)
    base = H.gpu_attention(w)
    perm = np.random.default_rng(1).permutation(w.num_pages)
    import copy
    w2 = copy.copy(w)
    w2.kv_pages = np.empty_like(w.kv_pages); w2.kv_pages[perm] = w.kv_pages
    w2.block_table = np.where(w.block_table >= 0, perm[np.maximum(w.block_table, 0)], -1).astype(np.int32)
    np.testing.assert_array_equal(H.gpu_attention(w2), base)


def _needle_case(P, E, Hq, Hkv, seed, n_needles):
    """Every chosen row scores one key ~22 above all others: out must be that value row."""
    w = W.make_uniform("needle", seed, 1, Hq, Hkv, P, E)
    N, PS, D = P + E, 16, 128
    nbits = max(int(N - 1).bit_length(), 1)
    t_all = np.arange(N)
    keys = np.zeros((N, D), np.float32)
    for b in range(nbits):
        keys[:, b] = np.where((t_all >> b) & 1, 8.0, -8.0)
    vals = np.zeros((N, D), np.float32)
    vals[:, 0] = t_all % 128; vals[:, 1] = (t_all // 128) % 128; vals[:, 2] = t_all // 16384
    vals[:, 3] = 1.0
    kb, vb = f32_to_bf16_bits(keys), f32_to_bf16_bits(vals)
    pages = w.block_table[0, t_all[:P] // PS]
    for g in range(Hkv):
        w.kv_pages[pages, 0, g, t_all[:P] % PS] = kb[:P]
        w.kv_pages[pages, 1, g, t_all[:P] % PS] = vb[:P]
        w.k_new[:, g] = kb[P:]; w.v_new[:, g] = vb[P:]
    rng = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([[0, E - 1], rng.integers(0, E, size=n_needles)]))
    targets = np.array([int(rng.integers(0, P + i + 1)) for i in rows])
    targets[0] = 0; targets[-1] = P + rows[-1]
    # q = key(target) * c with c chosen so that the winner leads by 2*8*8*c*scale = 24
    cq = 24.0 / (128.0 * w.softmax_scale)
    w.q[:] = 0
    for i, t in zip(rows, targets):
        w.q[i, :] = f32_to_bf16_bits(keys[t] * np.float32(cq))
    return w, rows, targets, bf16_bits_to_f32(vb).astype(np.float64)


def test_needle_small(H):
    w, rows, targets, vals = _needle_case(700, 300, 4, 2, 7, 64)
    got = bf16_bits_to_f32(H.gpu_attention(w)).astype(np.float64)
    for i, t in zip(rows, targets):
        # the losers leak ~1e-5 in total; a wrong page would be off by >= 1
        np.testing.assert_allclose(got[i], np.broadcast_to(vals[t], got[i].shape), rtol=0,
                                   atol=1e-3, err_msg=f"row {i} target {t}")
    # and the oracle agrees on what the needle rows hold
    want = oracle.attention_of(w, rows=rows.astype(np.int32))
    assert np.abs(want - vals[targets][:, None, :]).max() < 1e-6


def test_value_ones_and_key_shift(H):
    w = W.make_uniform("ones", 108, 1, 4, 2, 300, 200)
    one = f32_to_bf16_bits(np.float32(1.0))
    w.v_new[:] = one; w.kv_pages[:, 1] = one
    got = bf16_bits_to_f32(H.gpu_attention(w, num_splits=3)).astype(np.float64)
    assert np.abs(got - 1.0).max() <= 2 ** -7            # one bf16 ulp around 1
    # large common score offset: keys shifted by a constant vector (scores reach +-100)
    w = W.make_uniform("shift", 109, 1, 4, 2, 300, 200)
    kf = bf16_bits_to_f32(w.k_new); kf[..., :4] = 64.0; w.k_new = f32_to_bf16_bits(kf)
    pf = bf16_bits_to_f32(w.kv_pages[:, 0]); pf[..., :4] = 64.0; w.kv_pages[:, 0] = f32_to_bf16_bits(pf)
    _check(H.gpu_attention(w), oracle.attention_of(w), "key shift")


def _with_score_offsets(name, seed, P, E, offsets_of_key):
    """One request whose key j scores about offsets_of_key[j] (natural units, before the
    softmax) against every query row, on top of the N(0,1) noise of the other dimensions: the
    first four dimensions of every query are 8 and those of key j are offsets[j] / (32 scale)."""
    w = W.make_uniform(name, seed, 1, 4, 2, P, E)
    off = np.asarray(offsets_of_key, dtype=np.float32)
    assert off.shape == (P + E,)
    kval = off / np.float32(32.0 * w.softmax_scale)
    qf = bf16_bits_to_f32(w.q); qf[..., :4] = 8.0; w.q = f32_to_bf16_bits(qf)
    kf = bf16_bits_to_f32(w.k_new); kf[..., :4] = kval[P:, None, None]; w.k_new = f32_to_bf16_bits(kf)
    pf = bf16_bits_to_f32(w.kv_pages[:, 0])              # [page][head][slot][d]
    for j in range(P):
        pf[w.block_table[0, j // 16], :, j % 16, :4] = kval[j]
    w.kv_pages[:, 0] = f32_to_bf16_bits(pf)
    return w


# Score levels along the key sequence (natural units; times 1.44 in the exp2 domain of the
# kernel).  The row-tiled kernel keeps the reference exponent 0 while a row's maximum stays
# within 2^+-64, takes the row maximum as reference beyond that, and redoes a tile when a later
# key beats the reference by 2^80: every schedule below walks a different path through that.
_SCORE_SCHEDULES = {
    "mild": [-5, 5, 0, 8, -8, 3],
    "wide_but_plain": [-40, 40, -40, 0, 40, -20],
    "climb": [-120, -80, -50, 10, 90, 150],
    "descend": [150, 90, 10, -50, -80, -120],
    "all_very_negative": [-100, -101, -99, -100, -102, -100],
    "from_very_negative_into_the_plain_range": [-100, -100, -30, -30, 0, 0],
    "late_spike_beyond_the_plain_range": [0, 0, 0, 0, 60, 0],
    "swing_inside_the_plain_range": [-30, -30, -30, -30, 30, -30],
    "stale_reference_below_the_trigger": [-100, -100, -60, -60, -50, -100],
}


@pytest.mark.parametrize("splits", [1, 3])
@pytest.mark.parametrize("schedule", sorted(_SCORE_SCHEDULES))
def test_score_ranges_and_reference_changes(H, schedule, splits):
    P, E = 328, 200                                       # 9 key tiles, ragged on both sides
    levels = _SCORE_SCHEDULES[schedule]
    seg = -(-(P + E) // len(levels))
    off = np.repeat(np.asarray(levels, dtype=np.float32), seg)[:P + E]
    w = _with_score_offsets(f"scores_{schedule}", 130 + len(schedule), P, E, off)
    _check(H.gpu_attention(w, num_splits=splits), oracle.attention_of(w), f"{schedule} splits={splits}")


@pytest.mark.parametrize("case", ["row_tiled_ragged", "row_tiled_split", "packed_heads", "decode"])
def test_leftover_lds_contents_do_not_reach_the_result(H, case):
    """The kernels read only LDS they wrote in the same launch: the output bits do not depend on
    what an earlier kernel left in LDS, NaN and infinity patterns included."""
    import torch
    import paper_2511_03475_amd as cp
    if case == "row_tiled_ragged":
        w, ns = W.make_uniform("lds_a", 141, 3, 8, 2, [333, 0, 1000], [500, 700, 77]), 0
    elif case == "row_tiled_split":
        w, ns = W.make_uniform("lds_b", 142, 2, 4, 2, [2000, 900], [130, 300]), 3
    elif case == "packed_heads":
        w, ns = W.make_uniform("lds_c", 143, 4, 16, 2, [700, 300, 64, 1], [40, 100, 128, 9]), 1
    else:
        w, ns = W.make_uniform("lds_d", 144, 5, 16, 2, [3000, 1, 517, 64, 2048], [1, 2, 1, 4, 3]), 0
    case_ = H.DeviceCase(w, ns)
    stream = torch.cuda.current_stream()
    outs = []
    for pattern in (0x00000000, 0x7FC07FC0, 0xFFFFFFFF, 0x7F807F80, 0xFF80FF80, 0x3F803F80):
        case_.out.fill_(0x5555)
        cp.cp_probe_fill_lds(pattern, stream)
        case_.attention()
        outs.append(case_.out_bits().copy())
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])
    _check(outs[0], oracle.attention_of(w), f"lds leftovers {case}")


@pytest.mark.parametrize("tiles", range(1, 10))
def test_every_small_tile_count(H, tiles):
    """1 to 9 key tiles of 64 per work item, through the row-tiled kernel (num_splits = 1): the
    loop requests tiles two ahead and meets at a barrier after every second tile, so the first
    tiles, an odd and an even last tile and the cases without any prefetch are all here."""
    n = 64 * tiles
    for P, E in ((0, n - 10), (n - 7, 5), (n - 64, 64), (max(n - 100, 0), min(n, 100))):
        w = W.make_uniform(f"tiles{tiles}_{P}_{E}", 150 + tiles, 2, 4, 2, [P, max(P - 3, 0)], [E, E])
        _check(H.gpu_attention(w, num_splits=1), oracle.attention_of(w), f"tiles={tiles} P={P} E={E}")


def test_error_paths_return_codes(H):
    import paper_2511_03475_amd as cp
    w = W.make_uniform("err", 110, 1, 4, 2, 32, 32)
    case = H.DeviceCase(w, num_splits=2)
    args = (case.q, case.k_new, case.v_new, case.kv_pages, case.block_table, case.prefix_lens,
            case.extend_lens, case.out, None, case.shape)
    assert cp.cp_extend_attention(*args, None, 0, check=False) == cp.CP_ERR_WORKSPACE
    assert cp.cp_extend_attention(*args, case.workspace, case.ws_bytes - 1, check=False) == cp.CP_ERR_WORKSPACE
    assert cp.cp_extend_attention(None, *args[1:], case.workspace, case.ws_bytes, check=False) == cp.CP_ERR_NULL
    bad = cp.Shape(1, 4, 3, 128, 16, w.num_pages, w.max_pages_per_req, [32], [32], 0.1)
    assert cp.cp_extend_attention(*args[:-1], bad, None, 0, check=False) == cp.CP_ERR_SHAPE
    bad = cp.Shape(1, 4, 2, 64, 16, w.num_pages, w.max_pages_per_req, [32], [32], 0.1)
    assert cp.cp_write_kv(case.k_new, case.v_new, case.kv_pages, case.block_table,
                          case.prefix_lens, case.extend_lens, None, bad, check=False) == cp.CP_ERR_SHAPE
    bad = cp.Shape(1, 4, 2, 128, 16, w.num_pages, 1, [32], [32], 0.1)   # table too narrow
    assert cp.cp_extend_attention(*args[:-1], bad, None, 0, check=False) == cp.CP_ERR_SHAPE
    with pytest.raises(cp.CpError):
        cp.cp_extend_attention(*args, None, 0)


# ------------------------------------------------------------ scaled-down shapes of configs 2, 3
def test_config2_scaled_full_compare(H):
    w = W.config2_rag_fixed(batch=3, block=128, Hq=8, Hkv=2, query=32, cached_region_pages=256)
    _check(H.gpu_attention(w), oracle.attention_of(w), "config2 scaled")


def test_config3_scaled_full_compare(H):
    w = W.config3_rag_zipf(batch=12, block=64, topk=6, pool_ids=60, query=16, Hq=8, Hkv=2)
    assert max(w.notes["matched_blocks"]) >= 1
    _check(H.gpu_attention(w), oracle.attention_of(w), "config3 scaled")


def test_rag_batch_aligned_and_scheduled_by_the_context_index(H):
    """A small RAG batch whose block order and execution order come from the context index
    library (paper, Sections 4-5), then attention over the resulting aliased prefix pages."""
    import paper_2511_03475_amd as cp
    picks = W.rag_zipf_picks(seed=321, batch=12, topk=6, pool_ids=40)
    C = np.array(picks, np.int32)
    idx = cp.ContextIndex(C, np.full(len(picks), 6, np.int32), 0.001)
    aligned = [idx.aligned(i) for i in range(len(picks))]
    order = cp.cp_index_schedule([idx.path(i) for i in range(len(picks))])
    idx.close()
    w = W.rag_batch_from_blocks("rag_index", 321, aligned, block=64, query=16, Hq=8, Hkv=2, order=order)
    plain = W.rag_batch_from_blocks("rag_plain", 321, picks, block=64, query=16, Hq=8, Hkv=2)
    assert w.notes["token_hit_ratio"] > plain.notes["token_hit_ratio"]
    assert sum(w.notes["matched_blocks"]) > 0
    _check(H.gpu_attention(w), oracle.attention_of(w), "rag batch from the context index")


@pytest.mark.parametrize("B,P,E,G,Hkv", [
    (4, 2048, 1, 4, 2),       # decode: one new token, several heads packed into a workgroup
    (3, [4097, 15, 700], [1, 1, 1], 8, 1),
    (2, 3000, 16, 4, 2),      # a small chunk per request
    (1, 20000, 1, 4, 1),      # one long request: many splits
])
def test_decode_shapes(H, B, P, E, G, Hkv):
    """One or a few new tokens per request over a long cached prefix: wavefronts without valid
    rows only help loading, split-K fills the device."""
    w = W.make_uniform("decode", 131, B, G * Hkv, Hkv, P, E)
    want = oracle.attention_of(w)
    _check(H.gpu_attention(w), want, f"decode B={B} P={P} E={E}")
    _check(H.gpu_attention(w, num_splits=1), want, f"decode unsplit B={B} P={P} E={E}")


@pytest.mark.parametrize("G,Hkv,P,E", [
    (4, 2, [0, 0, 0], [1, 5, 16]),                 # no prefix at all: a single partly filled block
    (4, 2, [31, 32, 33, 1000], [1, 2, 3, 16]),     # blocks that straddle the prefix / suffix boundary
    (4, 2, [500, 7, 0, 4096], [9, 0, 11, 13]),     # a second row block that is partly filled; E = 0
    (8, 1, [777, 2048], [8, 3]),                   # G x E = 64 rows
    (1, 3, [100, 3000], [16, 1]),                  # one q head per KV head
    (2, 2, [65, 129], [7, 16]),
])
def test_decode_kernel_shapes(H, G, Hkv, P, E):
    """Calls with at most 64 rows per (request, KV head) run the wavefront-per-chunk kernel
    (cp_num_splits is then a multiple of 4); same bar against the oracle, and close to the
    row-tiled kernel on the same inputs."""
    import paper_2511_03475_amd as cp
    w = W.make_uniform("deck", 141, len(P), G * Hkv, Hkv, P, E)
    case = H.DeviceCase(w)
    assert cp.cp_num_splits(case.shape) % 4 == 0 and case.ws_bytes > 0
    want = oracle.attention_of(w)
    case.attention()
    got = case.out_bits()
    _check(got, want, f"decode kernel G={G} P={P} E={E}")
    case.attention()
    assert np.array_equal(case.out_bits(), got), "bitwise reproducible"
    tiled = bf16_bits_to_f32(H.gpu_attention(w, num_splits=1)).astype(np.float64)
    assert np.abs(bf16_bits_to_f32(got).astype(np.float64) - tiled).max() <= 2e-2


def test_decode_kernel_finds_a_needle_in_a_long_prefix(H):
    """One key far back in a 40k-token prefix dominates: every chunk but one contributes
    almost nothing and the merge must still return that key's value."""
    w = W.make_uniform("needle", 151, 2, 8, 2, [40000, 12345], [1, 2])
    q = bf16_bits_to_f32(w.q)
    pos = 23456
    page, slot = int(w.block_table[0, pos // 16]), pos % 16
    for kvh in range(2):
        # key = 4 * q of head 4 kvh (the first head of the group): score ~ 4 |q|^2 * scale >> others
        w.kv_pages[page, 0, kvh, slot, :] = f32_to_bf16_bits(4.0 * q[0, 4 * kvh, :])
    want = oracle.attention_of(w)
    got = H.gpu_attention(w)
    _check(got, want, "decode needle")
    v = bf16_bits_to_f32(w.kv_pages[page, 1, 0, slot, :]).astype(np.float64)
    assert np.abs(bf16_bits_to_f32(got)[0, 0].astype(np.float64) - v).max() < 5e-2


@pytest.mark.parametrize("max_e", [2, 40])
def test_large_batches_with_empty_requests(H, max_e):
    """More requests than one lookup step of 64 covers, many of them without extend tokens:
    every kernel finds the owner of a row or work unit by prefix sums over extend_lens
    (max_e = 2: decode-shaped kernel, max_e = 40: row-tiled kernel; cache write in both)."""
    rng = np.random.default_rng(4242 + max_e)
    B = 200
    E = rng.integers(0, max_e + 1, size=B)
    E[rng.random(B) < 0.3] = 0
    E[-1] = max_e
    P = rng.integers(0, 70, size=B)
    w = W.make_uniform("many", 4242 + max_e, B, 4, 2, [int(x) for x in P], [int(x) for x in E])
    _check(H.gpu_attention(w), oracle.attention_of(w), f"B={B} max_e={max_e}")
    case = H.DeviceCase(w)
    case.write_kv()
    np.testing.assert_array_equal(
        case.pool_bits(),
        oracle.write_kv(w.k_new, w.v_new, w.kv_pages, w.block_table, w.prefix_lens, w.extend_lens))


def _random_shape(rng):
    """One small random case: ragged batch, any GQA shape, lengths that straddle pages, key
    tiles, row tiles and the sizes at which the library changes kernel or head packing."""
    B = int(rng.integers(1, 6))
    Hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 4, 6, 8]))
    regime = rng.choice(["decode", "short", "mixed", "long", "long_prefix"])
    hiE = {"decode": 9, "short": 70, "mixed": 300, "long": 520, "long_prefix": 200}[regime]
    E = rng.integers(0 if regime == "mixed" else 1, hiE, size=B)
    P = rng.integers(0, 3000 if regime == "long_prefix" else 900, size=B)  # long: the steady-state loop
    P[rng.random(B) < 0.2] = 0
    snap = rng.random(B) < 0.3        # some lengths exactly on page / tile boundaries
    P[snap] = (P[snap] // 64) * 64
    if E.sum() == 0:
        E[0] = 1
    return B, G, Hkv, [int(x) for x in P], [int(x) for x in E]


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_attention_and_cache_write(H, seed):
    rng = np.random.default_rng(7700 + seed)
    B, G, Hkv, P, E = _random_shape(rng)
    w = W.make_uniform("fuzz", 7700 + seed, B, G * Hkv, Hkv, P, E, extra_table_cols=int(rng.integers(0, 3)))
    want = oracle.attention_of(w)
    what = f"seed={seed} B={B} G={G} Hkv={Hkv} P={P} E={E}"
    _check(H.gpu_attention(w), want, what + " auto")
    ns = int(rng.integers(1, 6))
    _check(H.gpu_attention(w, num_splits=ns), want, what + f" splits={ns}")
    case = H.DeviceCase(w)
    case.write_kv()
    np.testing.assert_array_equal(
        case.pool_bits(),
        oracle.write_kv(w.k_new, w.v_new, w.kv_pages, w.block_table, w.prefix_lens, w.extend_lens))


def _wide_random_shape(rng):
    """A wider draw than _random_shape: up to 70 requests, G up to 16, eight KV heads, long prefixes."""
    B = int(rng.choice([1, 2, 3, 5, 9, 70]))
    Hkv = int(rng.choice([1, 2, 3, 8]))
    G = int(rng.choice([1, 2, 3, 4, 6, 8, 16]))
    regime = rng.choice(["decode", "short", "mid", "long", "long_prefix"])
    hiE = {"decode": 6, "short": 70, "mid": 300, "long": 700, "long_prefix": 150}[regime]
    hiP = {"decode": 3000, "short": 900, "mid": 900, "long": 500, "long_prefix": 4000}[regime]
    if B == 70:
        hiE, hiP = min(hiE, 40), min(hiP, 300)
    E = rng.integers(0, hiE, size=B)
    P = rng.integers(0, hiP, size=B)
    if E.sum() == 0:
        E[0] = 1
    snap = rng.random(B) < 0.5
    P[snap] = (P[snap] // 64) * 64
    return B, G, Hkv, [int(x) for x in P], [int(x) for x in E]


@pytest.mark.parametrize("seed", range(32))
def test_wide_random_shapes_attention(H, seed):
    rng = np.random.default_rng(770000 + seed)
    B, G, Hkv, P, E = _wide_random_shape(rng)
    w = W.make_uniform("fuzz_wide", 770000 + seed, B, G * Hkv, Hkv, P, E)
    want = oracle.attention_of(w)
    what = f"seed={seed} B={B} G={G} Hkv={Hkv} P={P} E={E}"
    _check(H.gpu_attention(w), want, what + " auto")
    ns = int(rng.integers(1, 9))
    _check(H.gpu_attention(w, num_splits=ns), want, what + f" splits={ns}")
