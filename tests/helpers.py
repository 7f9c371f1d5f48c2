"""Small helpers for the tests: hand-built cases and an independent dense gather."""
import math

import numpy as np

from workloads import Workload, bf16_bits_to_f32, f32_to_bf16_bits


def case_from_floats(q, k_new, v_new, kv_pages, block_table, prefix_lens, extend_lens, scale=None):
    """Build a Workload from float arrays (rounded to bf16) and integer tables."""
    q = np.asarray(q, dtype=np.float32)
    k_new = np.asarray(k_new, dtype=np.float32)
    v_new = np.asarray(v_new, dtype=np.float32)
    kv_pages = np.asarray(kv_pages, dtype=np.float32)
    block_table = np.asarray(block_table, dtype=np.int32)
    T, Hq, D = q.shape
    Hkv = k_new.shape[1]
    return Workload(
        name="hand", batch=len(prefix_lens), num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D,
        page_size=kv_pages.shape[3], num_pages=kv_pages.shape[0],
        max_pages_per_req=block_table.shape[1],
        softmax_scale=(1.0 / math.sqrt(D)) if scale is None else scale,
        prefix_lens=np.asarray(prefix_lens, dtype=np.int32),
        extend_lens=np.asarray(extend_lens, dtype=np.int32), block_table=block_table,
        q=f32_to_bf16_bits(q), k_new=f32_to_bf16_bits(k_new), v_new=f32_to_bf16_bits(v_new),
        kv_pages=f32_to_bf16_bits(kv_pages))


def dense_kv(w, r):
    """Keys and values of request r as float64 [N, Hkv, D], gathered with numpy indexing.

    Written independently of the oracle's addressing code: token j < P lives in page
    block_table[r][j // PS] at slot j % PS; token j >= P is row cu[r] + j - P of k_new/v_new.
    """
    P, E = int(w.prefix_lens[r]), int(w.extend_lens[r])
    cu = int(w.cu_extend[r])
    pool = bf16_bits_to_f32(w.kv_pages).astype(np.float64)  # [pages, 2, Hkv, PS, D]
    tok = np.arange(P)
    pages = w.block_table[r][tok // w.page_size]
    slots = tok % w.page_size
    kp = pool[pages, 0, :, slots, :]  # [P, Hkv, D]
    vp = pool[pages, 1, :, slots, :]
    kn = bf16_bits_to_f32(w.k_new[cu:cu + E]).astype(np.float64)
    vn = bf16_bits_to_f32(w.v_new[cu:cu + E]).astype(np.float64)
    return np.concatenate([kp, kn], 0), np.concatenate([vp, vn], 0)


def error_stats(got_f64, want_f64):
    d = np.abs(np.asarray(got_f64, dtype=np.float64) - want_f64)
    rms = float(np.sqrt(np.mean(want_f64 ** 2))) if want_f64.size else 0.0
    return {"max_abs": float(d.max()) if d.size else 0.0,
            "mean_abs": float(d.mean()) if d.size else 0.0,
            "rel_rms": float(np.sqrt(np.mean(d ** 2)) / rms) if rms > 0 else 0.0,
            "n": int(d.size)}
