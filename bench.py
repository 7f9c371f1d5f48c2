#!/usr/bin/env python3
"""Benchmark of the extend-attention hot path on one MI355X.

One "step" = cp_write_kv (append the new K/V to the paged cache) followed by
cp_extend_attention (suffix rows attend to cached prefix + own keys) over one batch of seeded
synthetic input that is already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-extra] [--no-cpu]
                  [--operands normal|constant] [--splits N]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# HBM bytes per launch from two rocprofv3 --pmc runs (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, scale
# factors from a 1 GiB device copy in the same run), taken from the summaries under profiles/ and
# valid only for the kernel source they were taken with: reported as null as soon as that source
# changes.  They are not measured by this script.
TRAFFIC = {
    "source_sha256_16": "a2c80300eae4aaf4",
    "from": "profiles/extend_attn_kernel_long_context_32k.md, profiles/decode_attn_kernel_decode_b32_p10k.md",
    "long_context_32k": (2130379 * 2.0 + 524296) * 1024.0,      # extend_attn_kernel
    "decode_b32_p10k": (656155 * 2.0 + 4160) * 1024.0,          # decode_attn_kernel
}


def measured_traffic(workload: str):
    import hashlib
    src = os.path.join(ROOT, "paper_2511_03475_amd", "csrc", "cp_extend.hip")
    try:
        digest = hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]
    except OSError:
        return None
    if digest != TRAFFIC["source_sha256_16"]:
        return None
    return TRAFFIC.get(workload)


def roofline_of(workload: str, head: dict) -> dict:
    """Roofline entry of the dominant kernel: the matrix pipe when the call has more flops per
    algorithmic byte than the machine balance (2.5 PFLOP/s / 8 TB/s), HBM otherwise."""
    traffic = measured_traffic(workload)
    common = {"kernel": head["kernels"], "traffic": traffic,
              "traffic_source": TRAFFIC["from"] if traffic is not None else None,
              "avg_kernel_ms": head["attn_ms_avg"], "median_kernel_ms": head["attn_ms_median"]}
    if head["flops"] / head["alg_bytes_attn"] >= PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        return {"bound": "mfma", "achieved": head["tflops_attn"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": head["frac_mfma_peak"], **common}
    return {"bound": "hbm", "achieved": head["gbs_attn"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": head["frac_hbm_peak"], **common}


def _workload(name: str):
    import workloads as W
    table = {
        "tiny_extend": W.config1_tiny,
        "rag_fixed": W.config2_rag_fixed,
        # all 8 requests alias one cached 384-page prefix (the paper's multi-session case, Section 3.2)
        "rag_fixed_shared_prefix": lambda: W.config2_rag_fixed(shared_prefix=True),
        "rag_zipf": W.config3_rag_zipf,
        "long_context_32k": W.config4_long_context,
        "ctx128k_zero_reuse": lambda: W.config5_128k(False),
        "ctx128k_reuse": lambda: W.config5_128k(True),
        "short_extend_probe": W.probe_short_extend,
        "rag_zipf_context_index": rag_zipf_context_index,
        # decode shapes (one new token per request): the memory-bound end of the same path
        "decode_b32_p10k": lambda: W.make_uniform("decode_b32_p10k", W.BASE_SEED + 7, 32, 32, 8, 10240, 1),
        "decode_b32_p10k_e16": lambda: W.make_uniform("decode_b32_p10k_e16", W.BASE_SEED + 8, 32, 32, 8, 10240, 16),
        "decode_b1_p128k": lambda: W.make_uniform("decode_b1_p128k", W.BASE_SEED + 9, 1, 32, 8, 131072, 1),
        # one 2048-token chunk of a chunked prefill over 16k tokens already in the cache
        "chunked_prefill_b8_p16k_e2k": lambda: W.make_uniform("chunked_prefill_b8_p16k_e2k", W.BASE_SEED + 10, 8, 32, 8,
                                                              16384, 2048),
        "rag_zipf_as_retrieved": lambda: W.rag_batch_from_blocks("rag_zipf_as_retrieved", W.BASE_SEED + 3,
                                                                 W.rag_zipf_picks()),
    }
    return table[name]()


def index_align(picks, alpha: float = 0.001):
    """Aligned block orders and execution order of a batch from the context index library
    (construction, alignment and scheduling of the paper, Sections 4-5)."""
    import paper_2511_03475_amd as cp
    stride = max(len(p) for p in picks)
    C = np.full((len(picks), stride), -1, np.int32)
    L = np.zeros(len(picks), np.int32)
    for i, p in enumerate(picks):
        C[i, :len(p)] = p
        L[i] = len(p)
    idx = cp.ContextIndex(C, L, alpha)
    aligned = [idx.aligned(i) for i in range(len(picks))]
    order = cp.cp_index_schedule([idx.path(i) for i in range(len(picks))])
    idx.close()
    return aligned, order


def rag_zipf_context_index():
    """The rag_zipf batch (same retrieved blocks) with the block order and the execution order
    chosen by the context index instead of the frequency sort."""
    import workloads as W
    aligned, order = index_align(W.rag_zipf_picks())
    return W.rag_batch_from_blocks("rag_zipf_context_index", W.BASE_SEED + 3, aligned, order=order)


def algorithmic_bytes(w, with_cache_write: bool) -> float:
    """Bytes that must move once.  The attention call: q in, out, the new K/V read once, every
    prefix token's K/V once per request.  The whole step adds the cache append: the new K/V read
    and written once more."""
    T, Hq, Hkv, D = w.total_extend, w.num_q_heads, w.num_kv_heads, w.head_dim
    q_out = 2.0 * T * Hq * D * 2
    new_kv = T * Hkv * D * 2 * 2.0
    prefix = float(w.prefix_lens.astype(np.int64).sum()) * Hkv * D * 2 * 2
    return q_out + new_kv + prefix + (2.0 * new_kv if with_cache_write else 0.0)


class Runner:
    def __init__(self, w, num_splits: int = 0):
        import torch
        import paper_2511_03475_amd as cp
        self.torch, self.cp, self.w = torch, cp, w
        dev = "cuda:0"
        if OPERANDS == "constant":
            # every q, K and V element becomes bf16 1.0: same instructions and addresses, the
            # fewest toggling bits; shows what the power limit costs on N(0,1) operands
            for a in (w.q, w.k_new, w.v_new, w.kv_pages):
                a[...] = 0x3F80

        def up(a):
            a = np.ascontiguousarray(a)
            if a.dtype == np.uint16:
                a = a.view(np.int16)
            return torch.from_numpy(a).to(dev)

        self.q, self.k, self.v, self.pool = up(w.q), up(w.k_new), up(w.v_new), up(w.kv_pages)
        self.table, self.pl, self.el = up(w.block_table), up(w.prefix_lens), up(w.extend_lens)
        self.out = torch.empty_like(self.q)
        self.shape = cp.Shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.page_size,
                              w.num_pages, w.max_pages_per_req, w.prefix_lens, w.extend_lens,
                              w.softmax_scale, num_splits=num_splits)
        self.ws_bytes = cp.cp_workspace_bytes(self.shape)
        self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=dev)
        self.splits = cp.cp_num_splits(self.shape)
        self.kernels = cp.PLAN_KERNELS.get(cp.cp_plan_kind(self.shape), "?")

    def step(self, stream, ev=None):
        cp = self.cp
        cp.cp_write_kv(self.k, self.v, self.pool, self.table, self.pl, self.el, stream, self.shape)
        if ev is not None:
            ev[0].record(stream)
        cp.cp_extend_attention(self.q, self.k, self.v, self.pool, self.table, self.pl, self.el,
                               self.out, stream, self.shape, self.ws, self.ws_bytes)
        if ev is not None:
            ev[1].record(stream)

    def run(self, steps: int, warmup: int, settle_ms: float = 0.0):
        torch = self.torch
        stream = torch.cuda.current_stream()
        if settle_ms > 0:
            # The device clock dips a few ms after load begins and takes ~50 ms to reach its
            # steady value; short workloads would otherwise be timed inside that transient.
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            self.step(stream)
            torch.cuda.synchronize()
            one = max((time.perf_counter() - t0) * 1e3, 1e-3)
            for _ in range(min(2000, int(settle_ms / one) + 1)):
                self.step(stream)
        for _ in range(warmup):
            self.step(stream)
        events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                  for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(stream, events[i])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        attn_ms = [a.elapsed_time(b) for a, b in events]
        return (t1 - t0) * 1e3 / steps, attn_ms


SETTLE_MS = 100.0   # untimed run-in before the warm-up steps, see Runner.run
OPERANDS = "normal"  # "constant": see Runner.__init__


def measure(name: str, steps: int, warmup: int, num_splits: int = 0):
    t = time.perf_counter()
    w = _workload(name)
    gen_s = time.perf_counter() - t
    r = Runner(w, num_splits)
    ms_step, attn = r.run(steps, warmup, SETTLE_MS)
    attn_ms, attn_med, attn_min = float(np.mean(attn)), float(np.median(attn)), float(np.min(attn))
    flops = w.flops()
    b_attn, b_step = algorithmic_bytes(w, False), algorithmic_bytes(w, True)
    res = {
        "workload": name, "batch": w.batch, "q_heads": w.num_q_heads, "kv_heads": w.num_kv_heads,
        "prefix_tokens": int(w.prefix_lens.astype(np.int64).sum()), "extend_tokens": w.total_extend,
        "flops": flops, "splits": r.splits, "forced_splits": num_splits, "kernels": r.kernels, "steps": steps,
        "ms_per_step": ms_step, "attn_ms_avg": attn_ms, "attn_ms_median": attn_med, "attn_ms_min": attn_min,
        "tflops_step": flops / (ms_step * 1e-3) / 1e12,
        "tflops_attn": flops / (attn_ms * 1e-3) / 1e12,
        "frac_mfma_peak": flops / (attn_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "alg_bytes_attn": b_attn, "alg_bytes_step": b_step,
        "gbs_step": b_step / (ms_step * 1e-3) / 1e9,
        "gbs_attn": b_attn / (attn_ms * 1e-3) / 1e9,
        "frac_hbm_peak": b_attn / (attn_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "gen_s": gen_s,
    }
    if COPY_CEILING_GBS:
        res["frac_hbm_copy_ceiling"] = res["gbs_attn"] / COPY_CEILING_GBS
    if w.notes:
        res["notes"] = {k: v for k, v in w.notes.items()}
    return w, r, res


COPY_CEILING_GBS = None   # what a plain device-to-device copy moves on this device, set by main()


def measure_copy_ceiling(nbytes: int = 1 << 30, steps: int = 20) -> float:
    """GB/s (read + write) of a plain 1 GiB device-to-device copy kernel: the HBM rate this device
    gives a kernel that does nothing else, to put beside the published 8 TB/s."""
    import torch
    import paper_2511_03475_amd as cp
    a = torch.empty(nbytes // 4, dtype=torch.int32, device="cuda:0").fill_(1)
    b = torch.empty_like(a)
    stream = torch.cuda.current_stream()
    for _ in range(150):   # ~50 ms of the same load first, as for the workloads
        cp.cp_probe_copy(b, a, nbytes, stream)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    ev[0].record(stream)
    for i in range(steps):
        cp.cp_probe_copy(b, a, nbytes, stream)
        ev[i + 1].record(stream)
    torch.cuda.synchronize()
    ms = float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]))
    del a, b
    torch.cuda.empty_cache()
    return 2.0 * nbytes / (ms * 1e-3) / 1e9


def device_state() -> dict:
    """Clocks and power as rocm-smi prints them right after the timed runs.  The tool runs as a
    child process, started with this interpreter (no launcher hop); skipped under a profiler,
    whose preloaded library would initialise the GPU in the child as well.  Best effort: a note
    instead of figures when the tool is missing or refuses."""
    import shutil
    import subprocess
    if any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ) or "rocprof" in os.environ.get("LD_PRELOAD", ""):
        return {"skipped": "running under a profiler"}
    exe = shutil.which("rocm-smi") or "/opt/rocm/bin/rocm-smi"
    try:
        exe = os.path.realpath(exe)
        out = subprocess.run([sys.executable, exe, "--showclocks", "--showpower", "--json"], capture_output=True,
                             text=True, timeout=20)
        data = json.loads(out.stdout)
        card = data[sorted(data)[0]]
        return {k: v for k, v in card.items() if any(t in k.lower() for t in ("sclk", "mclk", "power", "fclk"))}
    except Exception as e:   # noqa: BLE001
        return {"unavailable": str(e)[:80]}


def cpu_baseline(w, budget_s: float = 15.0):
    """The fp64 oracle, as it stands, timed on a seeded row sample of the same workload."""
    import oracle
    rng = np.random.default_rng(12345)
    T = w.total_extend
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    cu = w.cu_extend

    def pairs_of(rows):
        rr = np.searchsorted(cu, rows, side="right") - 1
        return int((w.prefix_lens[rr].astype(np.int64) + (rows - cu[rr]) + 1).sum())

    probe = np.sort(rng.choice(T, size=min(T, max(threads // 4, 2)), replace=False)).astype(np.int32)
    t = time.perf_counter()
    oracle.attention_of(w, rows=probe)
    dt = time.perf_counter() - t
    per_pair = dt / max(pairs_of(probe), 1)
    mean_pairs = w.pairs_per_head() / max(T, 1)
    n = int(max(min(budget_s / max(per_pair * mean_pairs, 1e-9), T), 1))
    rows = np.sort(rng.choice(T, size=n, replace=False)).astype(np.int32)
    t = time.perf_counter()
    oracle.attention_of(w, rows=rows)
    dt = time.perf_counter() - t
    fl = 4.0 * w.head_dim * w.num_q_heads * pairs_of(rows)
    return {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} of {T} extend rows (seeded, all {w.num_q_heads} q heads), "
                      f"{dt:.1f} s of fp64 oracle; full workload extrapolates to "
                      f"{w.flops() / (fl / dt):.0f} s"}


PEAK_INT32_TOPS = 256 * 64 * 2.4e9 / 1e12   # 256 CUs x 64 lanes x 2.4 GHz, one 32-bit op per lane


def measure_context_distance(n: int = 8192, k: int = 15, stride: int = 16, steps: int = 20,
                             cpu: bool = True):
    """Pairwise context distance (paper, Eq. 1) for the index build: n contexts x top-k ids."""
    import torch
    import paper_2511_03475_amd as cp
    import workloads as W
    C, L = W.make_contexts(20251110, n, k, pool_ids=2000, stride=stride)
    dc, dl = torch.from_numpy(C).to("cuda:0"), torch.from_numpy(L).to("cuda:0")
    out = torch.empty((n, n), dtype=torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream()
    for _ in range(3):
        cp.cp_context_distance(dc, dl, n, stride, 0.001, out, stream)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    ev[0].record(stream)
    for i in range(steps):
        cp.cp_context_distance(dc, dl, n, stride, 0.001, out, stream)
        ev[i + 1].record(stream)
    torch.cuda.synchronize()
    ms = float(np.mean([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]))
    # Eq. 1 is symmetric and its own work is one comparison and one selection per pair of
    # positions of the k ids of two different contexts: n(n-1)/2 pairs x k^2 positions x 2.  The
    # kernel fills the whole matrix over the padded stride, i.e. it executes n^2 x stride^2 x 2.
    useful = 2.0 * (n * (n - 1) / 2.0) * k * k
    executed = 2.0 * n * n * stride * stride
    res = {"workload": f"context_distance n={n} k={k}", "ms": ms, "pairs_per_s": n * n / (ms * 1e-3),
           "roofline": {"bound": "alu", "achieved": useful / (ms * 1e-3) / 1e12, "peak": PEAK_INT32_TOPS,
                        "unit": "Tops/s (int32)", "frac": useful / (ms * 1e-3) / 1e12 / PEAK_INT32_TOPS,
                        "executed_tops": executed / (ms * 1e-3) / 1e12,
                        "frac_executed": executed / (ms * 1e-3) / 1e12 / PEAK_INT32_TOPS,
                        "traffic": None},
           "write_gbs": n * n * 4 / (ms * 1e-3) / 1e9}
    if cpu:
        import oracle
        m = n
        t = time.perf_counter()
        oracle.context_distance(C[:m], L[:m], 0.001)
        dt = time.perf_counter() - t
        res["cpu_baseline"] = {"value": m * m / dt, "unit": "pairs/s", "kind": "oracle",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
                               "sample": f"all {m} contexts ({m * m} pairs), {dt:.2f} s of fp64 oracle"}
    return res


def measure_context_index(n: int = 2000, k: int = 15, cpu: bool = True):
    """Index construction for n contexts of k retrieved blocks: Eq. 1 distances on the GPU,
    clustering / tree / alignment / schedule in the host library."""
    import torch
    import paper_2511_03475_amd as cp
    import workloads as W
    stride = 16
    C, L = W.make_contexts(20251111, n, k, pool_ids=2000, stride=stride)
    t0 = time.perf_counter()
    first_of, m = cp.cp_index_distinct(C, L)
    rows = np.zeros(m, np.int64)
    rows[first_of[::-1]] = np.arange(n)[::-1]            # first row of every distinct context
    dc, dl = torch.from_numpy(C[rows]).to("cuda:0"), torch.from_numpy(L[rows]).to("cuda:0")
    out = torch.empty((m, m), dtype=torch.float32, device="cuda:0")
    cp.cp_context_distance(dc, dl, m, stride, 0.001, out, torch.cuda.current_stream())
    D = out.cpu().numpy()
    t1 = time.perf_counter()
    idx = cp.ContextIndex(C, L, 0.001, dist=D)
    t2 = time.perf_counter()
    paths = [idx.path(i) for i in range(n)]
    order = cp.cp_index_schedule(paths)
    t3 = time.perf_counter()
    res = {"workload": f"context_index n={n} k={k}", "distinct": m, "nodes": idx.num_nodes(),
           "distance_gpu_incl_copies_s": t1 - t0, "cluster_tree_align_s": t2 - t1,
           "paths_schedule_s": t3 - t2, "total_s": t3 - t0, "contexts_per_s": n / (t3 - t0)}
    idx.close()
    assert sorted(order) == list(range(n))
    if cpu:
        from oracle import context_index as CI
        ns = 300
        sample = [list(map(int, C[i, :L[i]])) for i in range(ns)]
        t = time.perf_counter()
        ref = CI.ContextIndex.build(sample, 0.001)
        CI.schedule([ref.path(i) for i in range(ns)])
        dt = time.perf_counter() - t
        res["cpu_baseline"] = {"value": ns / dt, "unit": "contexts/s", "kind": "oracle", "cores": 1,
                               "sample": f"first {ns} of {n} contexts (cubic-time reference, {dt:.1f} s); "
                                         "not comparable at equal n"}
    return res


def measure_context_dedup(cpu: bool = True):
    """Multi-turn de-duplication (paper, Section 6) on a synthetic retrieval trace: host library,
    bytes of context per second and the share of bytes it removes."""
    import paper_2511_03475_amd as cp
    import workloads as W
    blocks, turns = W.make_conversation(20251112, turns=40, blocks_per_turn=12, pool_blocks=200,
                                        lines_per_block=200)
    total = sum(len(blocks[i]) for ids in turns for i in ids)
    conv = cp.Conversation(8)
    t = time.perf_counter()
    kept = 0
    for ids in turns:
        kept += conv.turn(ids, [blocks[i] for i in ids])[1]
    dt = time.perf_counter() - t
    conv.close()
    res = {"workload": f"context_dedup {len(turns)} turns x 12 blocks", "bytes": total, "kept_bytes": kept,
           "removed_fraction": 1.0 - kept / total, "seconds": dt, "mb_per_s": total / dt / 1e6,
           "ms_per_turn": dt / len(turns) * 1e3}
    if cpu:
        from oracle import context_dedup as OD
        ref = OD.Conversation(8)
        t = time.perf_counter()
        n = 0
        for ids in turns[:8]:
            n += sum(len(blocks[i]) for i in ids)
            ref.turn(ids, [blocks[i] for i in ids])
        dt = time.perf_counter() - t
        res["cpu_baseline"] = {"value": n / dt / 1e6, "unit": "MB/s", "kind": "oracle", "cores": 1,
                               "sample": f"first 8 of {len(turns)} turns ({n} bytes, {dt:.1f} s)"}
    return res


def measure_ceilings(iters: int = 100000):
    """What this device sustains on (a) nothing but back-to-back MFMAs and (b) the attention
    kernel's instruction mix per MFMA (operand read from LDS, softmax arithmetic) with nothing
    else in the way, on constant operands and on operands that toggle like N(0,1) samples: the
    device lowers its clock under a power limit, so the rates depend on the operand bits."""
    import torch
    import paper_2511_03475_amd as cp
    sink = torch.empty(cp.cp_probe_mfma_sink_floats(), dtype=torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream()
    out = {}
    for probe, fn in (("mfma_only", cp.cp_probe_mfma), ("attention_mix", cp.cp_probe_mix)):
        out[probe] = {}
        for name, kind in (("constant_operands", 0), ("normal_operands", 2)):
            for _ in range(10):   # ~200 ms of the same load first: steady clock, as for the workloads
                fn(kind, iters, sink, stream)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record(stream)
            for _ in range(3):
                fn(kind, iters, sink, stream)
            b.record(stream)
            torch.cuda.synchronize()
            out[probe][name] = 3.0 * cp.cp_probe_mfma_flops(iters) / (a.elapsed_time(b) * 1e-3) / 1e12
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="long_context_32k")
    ap.add_argument("--no-extra", action="store_true", help="skip the other workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--settle-ms", type=float, default=SETTLE_MS,
                    help="untimed run-in of each workload before its warm-up steps (clock transient)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for HBM counters)")
    ap.add_argument("--operands", choices=("normal", "constant"), default="normal",
                    help="constant: q, K, V all bf16 1.0 (same work, least power; for the clock account)")
    ap.add_argument("--splits", type=int, default=0, help="force the split-K factor of the headline workload")
    args = ap.parse_args()
    globals()["SETTLE_MS"] = args.settle_ms
    globals()["OPERANDS"] = args.operands
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only; use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2511_03475_amd as cp
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    cp.load_library()   # raises if the HIP library has not been built

    if args.copy_probe:
        a = torch.empty(1 << 28, dtype=torch.int32, device="cuda:0").fill_(1)
        b = torch.empty_like(a)
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()

    if args.workload == "context_distance":   # the distance kernel alone (for profiling it)
        print(json.dumps(measure_context_distance(steps=args.steps, cpu=not args.no_cpu)))
        return

    globals()["COPY_CEILING_GBS"] = measure_copy_ceiling()
    w, r, head = measure(args.workload, args.steps, args.warmup, args.splits)
    cpu = None if args.no_cpu else cpu_baseline(w)
    del r
    torch.cuda.empty_cache()

    extra = []
    if not args.no_extra:
        for name in ("tiny_extend", "rag_fixed", "rag_fixed_shared_prefix", "rag_zipf", "rag_zipf_as_retrieved",
                     "rag_zipf_context_index", "long_context_32k", "long_context_32k:split2", "ctx128k_zero_reuse",
                     "ctx128k_reuse", "short_extend_probe", "chunked_prefill_b8_p16k_e2k",
                     "decode_b32_p10k", "decode_b32_p10k_e16", "decode_b1_p128k"):
            if name == args.workload and args.splits == 0:
                extra.append({k: head[k] for k in head})
                continue
            steps = 5 if name.startswith("ctx128k") or name.startswith("rag_zipf") else 20
            # "name:splitN": the same workload with the keys split N ways by force (long_context_32k
            # is timed with the split off, which the plan chooses and which is faster, and on)
            base, _, forced = name.partition(":split")
            _, rr, res = measure(base, steps, 2, int(forced) if forced else 0)
            res["workload"] = name
            extra.append(res)
            del rr
            torch.cuda.empty_cache()
    by = {e["workload"]: e for e in extra}
    reuse = None
    if "ctx128k_zero_reuse" in by and "ctx128k_reuse" in by:
        reuse = {"measured_step": by["ctx128k_zero_reuse"]["ms_per_step"] / by["ctx128k_reuse"]["ms_per_step"],
                 "measured_attn": by["ctx128k_zero_reuse"]["attn_ms_avg"] / by["ctx128k_reuse"]["attn_ms_avg"],
                 "algorithmic_flop_ratio": by["ctx128k_zero_reuse"]["flops"] / by["ctx128k_reuse"]["flops"],
                 "token_ratio": 8.0}

    line = {
        "metric": "extend-attention TFLOP/s and % of bf16 MFMA peak at 32k/128k ctx",
        "value": head["tflops_step"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "clock_settle_ms": args.settle_ms, "operands": args.operands,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "batch": head["batch"], "q_heads": head["q_heads"],
                   "kv_heads": head["kv_heads"], "head_dim": 128, "page_size": 16,
                   "prefix_tokens": head["prefix_tokens"], "extend_tokens": head["extend_tokens"],
                   "step": "cp_write_kv + cp_extend_attention", "splits": head["splits"]},
        "roofline": roofline_of(args.workload, head),
        "cpu_baseline": cpu,
        "hbm_copy_ceiling_gbs": COPY_CEILING_GBS,
        "device_state_after": device_state(),
    }
    if extra:
        line["workloads"] = [{k: (round(v, 4) if isinstance(v, float) else v) for k, v in e.items()
                              if k not in ("notes",)} for e in extra]
        line["rag_zipf_hit_ratio"] = {name: by[name]["notes"]["token_hit_ratio"]
                                      for name in ("rag_zipf_as_retrieved", "rag_zipf", "rag_zipf_context_index")
                                      if name in by and "notes" in by[name]}
    if reuse:
        line["reuse_speedup_128k"] = reuse
    if not args.no_extra:
        line["context_distance"] = measure_context_distance(cpu=not args.no_cpu)
        line["context_index"] = measure_context_index(cpu=not args.no_cpu)
        line["context_dedup"] = measure_context_dedup(cpu=not args.no_cpu)
        ceil = measure_ceilings()
        line["measured_ceilings_tflops"] = ceil
        if line["roofline"]["bound"] == "mfma":
            line["roofline"]["frac_of_measured_mfma_ceiling"] = head["tflops_attn"] / ceil["mfma_only"]["normal_operands"]
            line["roofline"]["frac_of_measured_mix_ceiling"] = head["tflops_attn"] / ceil["attention_mix"]["normal_operands"]
    print(json.dumps(line))


if __name__ == "__main__":
    main()
