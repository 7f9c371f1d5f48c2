"""Seeded synthetic inputs for prefix-cached "extend" prefill attention.

This module only draws random numbers and builds integer tables.  It holds none
of the arithmetic of attention or of the cache write: it is the single producer
of inputs for both the CPU oracle and the GPU library, so that the two are
always compared on identical bits.

Shapes follow the workloads of the paper's setting (Section 2.2, Section 5):
context blocks of 1024 tokens, top-k retrieval with k around 10-15, prompts of
20k-130k tokens, heavy-tailed block popularity, GQA head shapes of 32B/70B-class
models.  The paper's datasets and model weights are not used; values are i.i.d.
N(0,1) rounded once to bf16 because the cost of attention does not depend on the
values.

Array conventions (all numpy, bf16 carried as raw uint16 bit patterns):
  q              [T, Hq,  D]   packed extend rows, T = sum(extend_lens)
  k_new, v_new   [T, Hkv, D]
  kv_pages       [num_pages, 2, Hkv, PS, D]   index 0 = K, 1 = V
  block_table    [B, max_pages_per_req] int32, -1 where unused
  prefix_lens, extend_lens [B] int32
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional

import numpy as np

HEAD_DIM = 128
PAGE_SIZE = 16
BASE_SEED = 20251103


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even), returned as uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(rng: np.random.Generator, shape, chunk_elems: int = 1 << 23,
                threads: int = 8) -> np.ndarray:
    """N(0,1) drawn in float32 and rounded once to bf16.

    The array is cut into fixed chunks, each filled from its own child generator, so the
    result depends only on the seed and the shape, not on how many threads fill it.
    """
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.uint16)
    nchunks = (n + chunk_elems - 1) // chunk_elems
    if nchunks == 0:
        return out.reshape(shape)
    children = rng.spawn(nchunks)

    def fill(c):
        lo = c * chunk_elems
        hi = min(lo + chunk_elems, n)
        out[lo:hi] = f32_to_bf16_bits(children[c].standard_normal(hi - lo, dtype=np.float32))

    if nchunks == 1 or threads <= 1:
        for c in range(nchunks):
            fill(c)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(nchunks)))
    return out.reshape(shape)


def normal_bf16_rows(rng: np.random.Generator, shape, row_lo: int, row_hi: int,
                     chunk_elems: int = 1 << 23, threads: int = 8) -> np.ndarray:
    """Rows [row_lo, row_hi) of normal_bf16(rng, shape), without drawing the other rows: only the
    chunks that overlap the slice are filled (chunk c always comes from child generator c)."""
    n = int(np.prod(shape, dtype=np.int64))
    row = n // int(shape[0])
    lo, hi = row_lo * row, row_hi * row
    nchunks = (n + chunk_elems - 1) // chunk_elems
    children = rng.spawn(nchunks)
    out = np.empty(hi - lo, dtype=np.uint16)

    def fill(c):
        c_lo, c_hi = c * chunk_elems, min((c + 1) * chunk_elems, n)
        vals = f32_to_bf16_bits(children[c].standard_normal(c_hi - c_lo, dtype=np.float32))
        a, b = max(c_lo, lo), min(c_hi, hi)
        out[a - lo:b - lo] = vals[a - c_lo:b - c_lo]

    todo = [c for c in range(nchunks) if c * chunk_elems < hi and min((c + 1) * chunk_elems, n) > lo]
    if len(todo) <= 1 or threads <= 1:
        for c in todo:
            fill(c)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, todo))
    return out.reshape((row_hi - row_lo,) + tuple(shape[1:]))


@dataclasses.dataclass
class Workload:
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    num_pages: int
    max_pages_per_req: int
    softmax_scale: float
    prefix_lens: np.ndarray
    extend_lens: np.ndarray
    block_table: np.ndarray
    q: np.ndarray
    k_new: np.ndarray
    v_new: np.ndarray
    kv_pages: np.ndarray
    notes: dict = dataclasses.field(default_factory=dict)

    @property
    def total_extend(self) -> int:
        return int(self.extend_lens.sum())

    @property
    def cu_extend(self) -> np.ndarray:
        cu = np.zeros(self.batch + 1, dtype=np.int64)
        np.cumsum(self.extend_lens, out=cu[1:])
        return cu

    def pairs_per_head(self) -> int:
        """Number of (query row, visible key) combinations for one q head."""
        p = self.prefix_lens.astype(np.int64)
        e = self.extend_lens.astype(np.int64)
        return int((e * p + e * (e + 1) // 2).sum())

    def flops(self) -> float:
        """Algorithmic flops: 2*D for QK^T plus 2*D for PV per visible pair and q head."""
        return 4.0 * self.head_dim * self.num_q_heads * self.pairs_per_head()


def _streams(seed: int):
    """Independent sub-streams in the fixed order q, k_new, v_new, pool, pages, structure."""
    return np.random.default_rng(seed).spawn(6)


def _assemble(name, seed, Hq, Hkv, prefix_lens, extend_lens, block_table, num_pages,
              rngs=None, notes=None, fill_pool=True) -> Workload:
    rq, rk, rv, rpool, _, _ = rngs if rngs is not None else _streams(seed)
    prefix_lens = np.asarray(prefix_lens, dtype=np.int32)
    extend_lens = np.asarray(extend_lens, dtype=np.int32)
    T = int(extend_lens.sum())
    D, PS = HEAD_DIM, PAGE_SIZE
    q = normal_bf16(rq, (T, Hq, D))
    k_new = normal_bf16(rk, (T, Hkv, D))
    v_new = normal_bf16(rv, (T, Hkv, D))
    if fill_pool:
        kv_pages = normal_bf16(rpool, (num_pages, 2, Hkv, PS, D))
    else:
        kv_pages = np.zeros((num_pages, 2, Hkv, PS, D), dtype=np.uint16)
    return Workload(
        name=name, batch=len(prefix_lens), num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D,
        page_size=PS, num_pages=num_pages, max_pages_per_req=block_table.shape[1],
        softmax_scale=1.0 / math.sqrt(D), prefix_lens=prefix_lens, extend_lens=extend_lens,
        block_table=np.ascontiguousarray(block_table, dtype=np.int32),
        q=q, k_new=k_new, v_new=v_new, kv_pages=kv_pages, notes=notes or {})


def make_uniform(name: str, seed: int, batch: int, Hq: int, Hkv: int, prefix_len, extend_len,
                 num_pages: Optional[int] = None, extra_table_cols: int = 0,
                 fill_pool: bool = True) -> Workload:
    """Requests with given prefix/extend lengths (scalars or per-request lists).

    Every request owns ceil((P+E)/PS) distinct physical pages, placed by one seeded
    permutation of the pool.
    """
    rngs = _streams(seed)
    P = np.broadcast_to(np.asarray(prefix_len, dtype=np.int64), (batch,)).copy()
    E = np.broadcast_to(np.asarray(extend_len, dtype=np.int64), (batch,)).copy()
    need = (P + E + PAGE_SIZE - 1) // PAGE_SIZE
    total = int(need.sum())
    if num_pages is None:
        num_pages = max(total, 1)
    assert num_pages >= total, "pool too small"
    perm = rngs[4].permutation(num_pages)
    width = max(int(need.max()) if batch else 0, 1) + extra_table_cols
    table = np.full((batch, width), -1, dtype=np.int32)
    pos = 0
    for r in range(batch):
        table[r, :need[r]] = perm[pos:pos + need[r]]
        pos += int(need[r])
    return _assemble(name, seed, Hq, Hkv, P, E, table, num_pages, rngs=rngs, fill_pool=fill_pool)


def config1_tiny(seed: int = BASE_SEED + 1) -> Workload:
    """1 request, 8 q heads / 2 KV heads, P=512 (32 pages), E=128, 64-page pool."""
    return make_uniform("tiny_extend", seed, 1, 8, 2, 512, 128, num_pages=64)


def config2_rag_fixed(seed: int = BASE_SEED + 2, batch: int = 8, block: int = 1024,
                      cached_blocks: int = 6, total_blocks: int = 8, query: int = 256,
                      Hq: int = 32, Hkv: int = 8, cached_region_pages: int = 4096,
                      shared_prefix: bool = False) -> Workload:
    """RAG batch with fixed reuse.

    Cached pages are a seeded permutation inside a region of `cached_region_pages`
    pages; the destination pages of the extend part come from a seeded permutation
    of a second region appended after it (the stated pool cannot hold both).
    shared_prefix: every request's cached prefix is the same physical pages (the paper's
    multi-session case, Section 3.2: sessions that share one cached context).
    """
    rngs = _streams(seed)
    P = cached_blocks * block
    E = (total_blocks - cached_blocks) * block + query
    assert P % PAGE_SIZE == 0
    pp = P // PAGE_SIZE
    ep = (E + PAGE_SIZE - 1) // PAGE_SIZE
    assert batch * pp <= cached_region_pages
    perm_c = rngs[4].permutation(cached_region_pages)
    perm_e = cached_region_pages + rngs[4].permutation(batch * ep)
    table = np.full((batch, pp + ep), -1, dtype=np.int32)
    for r in range(batch):
        table[r, :pp] = perm_c[:pp] if shared_prefix else perm_c[r * pp:(r + 1) * pp]
        table[r, pp:pp + ep] = perm_e[r * ep:(r + 1) * ep]
    return _assemble("rag_fixed_shared_prefix" if shared_prefix else "rag_fixed", seed, Hq, Hkv, [P] * batch, [E] * batch, table,
                     cached_region_pages + batch * ep, rngs=rngs)


def rag_zipf_picks(seed: int = BASE_SEED + 3, batch: int = 32, topk: int = 10,
                   pool_ids: int = 2000, zipf_s: float = 1.1) -> List[List[int]]:
    """The retrieved block ids of a RAG batch, in retrieval order: each request draws `topk`
    distinct ids with weight rank^-s."""
    rs = _streams(seed)[5]
    w = (np.arange(pool_ids, dtype=np.float64) + 1.0) ** (-zipf_s)
    w /= w.sum()
    return [[int(i) for i in rs.choice(pool_ids, size=topk, replace=False, p=w)] for _ in range(batch)]


def rag_batch_from_blocks(name: str, seed: int, contexts: List[List[int]], block: int = 1024,
                          query: int = 128, Hq: int = 32, Hkv: int = 8,
                          order: Optional[List[int]] = None) -> Workload:
    """A RAG batch whose requests are given as block-id sequences, as they will be run.

    Request r of the batch is contexts[order[r]] (order: execution order, default as given).
    Its cached prefix is the longest leading block sequence it shares with any earlier request
    of the batch (an exact prefix cache that has kept them all), and its prefix pages alias
    that request's physical pages.  Every request ends with `query` extra tokens.
    """
    order = list(range(len(contexts))) if order is None else [int(i) for i in order]
    assert sorted(order) == list(range(len(contexts)))
    rngs = _streams(seed)
    seqs = [contexts[i] for i in order]
    batch = len(seqs)
    assert block % PAGE_SIZE == 0
    bp = block // PAGE_SIZE
    pages_of = [(len(c) * block + query + PAGE_SIZE - 1) // PAGE_SIZE for c in seqs]
    matched, donor = [], []
    for r in range(batch):
        best, who = 0, -1
        for e in range(r):
            m = 0
            while m < len(seqs[r]) and m < len(seqs[e]) and seqs[r][m] == seqs[e][m]:
                m += 1
            if m > best:
                best, who = m, e
        matched.append(best)
        donor.append(who)
    fresh = [pages_of[r] - matched[r] * bp for r in range(batch)]
    num_pages = int(sum(fresh))
    perm = rngs[4].permutation(num_pages)
    table = np.full((batch, max(pages_of)), -1, dtype=np.int32)
    pos = 0
    for r in range(batch):
        a = matched[r] * bp
        if a:
            table[r, :a] = table[donor[r], :a]
        table[r, a:pages_of[r]] = perm[pos:pos + fresh[r]]
        pos += fresh[r]
    P = [m * block for m in matched]
    E = [(len(seqs[r]) - matched[r]) * block + query for r in range(batch)]
    hit = float(sum(P)) / float(sum(P) + sum(E))
    return _assemble(name, seed, Hq, Hkv, P, E, table, num_pages, rngs=rngs,
                     notes={"matched_blocks": matched, "token_hit_ratio": hit, "order": order})


def config3_rag_zipf(seed: int = BASE_SEED + 3, batch: int = 32, block: int = 1024,
                     topk: int = 10, pool_ids: int = 2000, zipf_s: float = 1.1,
                     query: int = 128, Hq: int = 32, Hkv: int = 8) -> Workload:
    """RAG batch with Zipf block popularity and frequency-sorted block order: the blocks of
    each request are reordered by descending count over the batch (ties: smaller id first)."""
    picks = rag_zipf_picks(seed, batch, topk, pool_ids, zipf_s)
    counts = np.bincount(np.concatenate([np.asarray(p) for p in picks]), minlength=pool_ids)
    aligned = [sorted(p, key=lambda i: (-int(counts[i]), i)) for p in picks]
    return rag_batch_from_blocks("rag_zipf", seed, aligned, block, query, Hq, Hkv)


def config4_long_context(seed: int = BASE_SEED + 4, batch: int = 4, prefix: int = 24576,
                         extend: int = 8192, Hq: int = 64, Hkv: int = 8) -> Workload:
    """One layer of a 70B-class GQA model at 32k context, 75 % cached."""
    w = make_uniform("long_context_32k", seed, batch, Hq, Hkv, prefix, extend)
    return w


def config5_128k(reuse: bool, seed: int = BASE_SEED + 5, total: int = 131072,
                 cached: int = 114688, Hq: int = 32, Hkv: int = 8) -> Workload:
    """One 128k-token request: zero reuse (full causal prefill) or 87.5 % reuse.

    Both runs see the same token streams: the reuse run's q / k_new / v_new are the last
    total - cached rows of the zero-reuse run's, its cached pages hold the K/V of the first
    `cached` rows, and the block tables are equal.  The reuse run's output therefore equals the
    last rows of the zero-reuse run's output up to rounding.
    """
    if not reuse:
        return make_uniform("ctx128k_zero_reuse", seed, 1, Hq, Hkv, 0, total, fill_pool=False)
    rq, rk, rv, _, rpages, _ = _streams(seed)
    D, PS = HEAD_DIM, PAGE_SIZE
    assert cached % PS == 0 and 0 < cached < total
    num_pages = (total + PS - 1) // PS
    table = rpages.permutation(num_pages).astype(np.int32)[None, :]      # as make_uniform places them
    q = normal_bf16_rows(rq, (total, Hq, D), cached, total)
    k_all_lo = normal_bf16_rows(rk, (total, Hkv, D), 0, cached)
    v_all_lo = normal_bf16_rows(rv, (total, Hkv, D), 0, cached)
    _, rk, rv, _, _, _ = _streams(seed)       # a generator hands out its children only once
    k_new = normal_bf16_rows(rk, (total, Hkv, D), cached, total)
    v_new = normal_bf16_rows(rv, (total, Hkv, D), cached, total)
    kv_pages = np.zeros((num_pages, 2, Hkv, PS, D), dtype=np.uint16)
    pp = cached // PS
    kv_pages[table[0, :pp], 0] = k_all_lo.reshape(pp, PS, Hkv, D).transpose(0, 2, 1, 3)
    kv_pages[table[0, :pp], 1] = v_all_lo.reshape(pp, PS, Hkv, D).transpose(0, 2, 1, 3)
    return Workload(
        name="ctx128k_reuse", batch=1, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, page_size=PS,
        num_pages=num_pages, max_pages_per_req=num_pages, softmax_scale=1.0 / math.sqrt(D),
        prefix_lens=np.array([cached], np.int32), extend_lens=np.array([total - cached], np.int32),
        block_table=np.ascontiguousarray(table), q=q, k_new=k_new, v_new=v_new, kv_pages=kv_pages,
        notes={"shares_streams_with": "ctx128k_zero_reuse"})


def probe_short_extend(seed: int = BASE_SEED + 6, batch: int = 32, prefix: int = 10240,
                       extend: int = 128, Hq: int = 32, Hkv: int = 8) -> Workload:
    """Memory-bound short-extend case: a fully cached RAG request (query only)."""
    return make_uniform("short_extend_probe", seed, batch, Hq, Hkv, prefix, extend)


def sample_rows(w: Workload, seed: int, q_block: int = 128, edge: int = 16,
                seams: int = 16, extra_boundaries: Optional[List[int]] = None) -> np.ndarray:
    """Seeded sample of packed extend rows for sampled parity at large sizes.

    Per request: one random row in every q_block-row block, the first and last `edge`
    rows, rows around `seams` random block seams, and rows around given boundaries.
    Returns sorted unique packed row indices (int32).
    """
    rng = np.random.default_rng(seed)
    cu = w.cu_extend
    rows = []
    for r in range(w.batch):
        E = int(w.extend_lens[r])
        if E == 0:
            continue
        nb = (E + q_block - 1) // q_block
        starts = np.arange(nb, dtype=np.int64) * q_block
        ends = np.minimum(starts + q_block, E)
        loc = [starts + (rng.random(nb) * (ends - starts)).astype(np.int64)]
        loc.append(np.arange(min(edge, E)))
        loc.append(np.arange(max(E - edge, 0), E))
        if nb > 1:
            s = rng.integers(1, nb, size=min(seams, nb - 1)) * q_block
            loc += [s - 1, s, s + 1]
        for b in (extra_boundaries or []):
            loc.append(np.array([b - 1, b, b + 1]))
        allr = np.concatenate(loc)
        allr = allr[(allr >= 0) & (allr < E)]
        rows.append(cu[r] + allr)
    if not rows:
        return np.zeros(0, dtype=np.int32)
    return np.unique(np.concatenate(rows)).astype(np.int32)


def make_contexts(seed: int, n: int, k, pool_ids: int = 2000, zipf_s: float = 1.1,
                  stride: Optional[int] = None):
    """Contexts for the context index (paper, Section 4.1): n ordered lists of distinct block ids.

    Each context draws its ids without replacement with weight rank^-s (heavy-tailed block
    popularity); the draw order stands for the retriever's relevance order.  k is the number of
    blocks per context (an int, or a (lo, hi) range drawn uniformly per context).
    Returns (contexts [n, stride] int32 padded with -1, lens [n] int32).
    """
    rng = np.random.default_rng(seed)
    if isinstance(k, int):
        lens = np.full(n, k, dtype=np.int32)
    else:
        lens = rng.integers(k[0], k[1] + 1, size=n).astype(np.int32)
    kmax = int(lens.max()) if n else 0
    stride = stride or max(kmax, 1)
    assert stride >= kmax and pool_ids >= kmax
    w = (np.arange(pool_ids, dtype=np.float64) + 1.0) ** (-zipf_s)
    # Gumbel top-k: the kmax largest perturbed log-weights, in order, are a draw without
    # replacement with probabilities proportional to w
    contexts = np.full((n, stride), -1, dtype=np.int32)
    logw = np.log(w)
    chunk = 4096
    for lo in range(0, n, chunk):
        hi = min(lo + chunk, n)
        g = logw[None, :] + rng.gumbel(size=(hi - lo, pool_ids))
        top = np.argsort(-g, axis=1)[:, :kmax].astype(np.int32)
        contexts[lo:hi, :kmax] = top
    for i in range(n):
        contexts[i, lens[i]:] = -1
    return contexts, lens


def make_conversation(seed: int, turns: int = 6, blocks_per_turn: int = 8, pool_blocks: int = 24,
                      lines_per_block: int = 40, shared_sections: int = 10,
                      section_prob: float = 0.35):
    """Synthetic multi-turn retrieval trace for the de-duplication path: text blocks whose lines
    are random words, with template sections (runs of 3-8 lines) shared between blocks, and turns
    that retrieve overlapping sets of block ids (Zipf over the pool).  Stands in for the
    multi-turn retrieval traces of the paper's datasets.

    Returns (blocks: dict id -> bytes, turns: list of lists of ids).
    """
    rng = np.random.default_rng(seed)

    def line() -> bytes:
        words = ["".join(chr(97 + int(c)) for c in rng.integers(0, 26, size=int(rng.integers(2, 10))))
                 for _ in range(int(rng.integers(4, 13)))]
        return (" ".join(words) + "\n").encode()

    sections = [b"".join(line() for _ in range(int(rng.integers(3, 9)))) for _ in range(shared_sections)]
    blocks = {}
    for b in range(pool_blocks):
        parts, n = [], 0
        while n < lines_per_block:
            if shared_sections and rng.random() < section_prob / 4:
                s = sections[int(rng.integers(0, shared_sections))]
                parts.append(s)
                n += s.count(b"\n")
            else:
                parts.append(line())
                n += 1
        text = b"".join(parts)
        if b % 3 == 0:
            text = text[:-1]                 # some blocks end without a newline
        blocks[b] = text
    w = (np.arange(pool_blocks, dtype=np.float64) + 1.0) ** -1.1
    w /= w.sum()
    seq = [[int(i) for i in rng.choice(pool_blocks, size=min(blocks_per_turn, pool_blocks), replace=False, p=w)]
           for _ in range(turns)]
    return blocks, seq
