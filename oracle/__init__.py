"""ctypes front end of the fp64 CPU oracle (extend_attention_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the CPU-baseline
leg of the benchmark.  The GPU library and its Python binding never import this package,
and this package imports nothing from them.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "extend_attention_oracle.c"),
         os.path.join(_HERE, "context_distance_oracle.c")]
_LIB = os.path.join(_HERE, "libcp_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (plain C + OpenMP)."""
    if force or not os.path.exists(_LIB) or \
            os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               *_SRCS, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.oracle_extend_attention.restype = ctypes.c_int
        lib.oracle_extend_attention.argtypes = [
            u16p, u16p, u16p, u16p, i32p, i32p, i32p,
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
            ctypes.c_int32, ctypes.c_double, i32p, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_int64, f64p, f64p]
        lib.oracle_write_kv.restype = ctypes.c_int
        lib.oracle_write_kv.argtypes = [
            u16p, u16p, u16p, i32p, i32p, i32p,
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        lib.oracle_context_distance.restype = ctypes.c_int
        lib.oracle_context_distance.argtypes = [i32p, i32p, ctypes.c_int32, ctypes.c_int32,
                                                ctypes.c_double, f64p]
        _lib = lib
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def extend_attention(q, k_new, v_new, kv_pages, block_table, prefix_lens, extend_lens,
                     softmax_scale: float, rows: Optional[np.ndarray] = None,
                     key_lo: int = 0, key_hi: int = -1, return_lse: bool = False):
    """fp64 attention of the extend rows over cached prefix + own keys.

    q [T,Hq,D], k_new/v_new [T,Hkv,D], kv_pages [num_pages,2,Hkv,PS,D] as uint16 bf16 bits;
    block_table [B,max_pages] int32; prefix_lens/extend_lens [B] int32.
    rows: packed row indices to compute (default: all).  key_lo/key_hi restrict the keys of
    every row to that range (default: all visible keys).
    Returns out [n_rows,Hq,D] float64 (and lse [n_rows,Hq] if requested).
    """
    lib = _load()
    q, qp = _u16(q)
    k_new, kp = _u16(k_new)
    v_new, vp = _u16(v_new)
    kv_pages, pp = _u16(kv_pages)
    block_table, tp = _i32(block_table)
    prefix_lens, plp = _i32(prefix_lens)
    extend_lens, elp = _i32(extend_lens)
    B = prefix_lens.shape[0]
    T, Hq, D = q.shape
    Hkv = k_new.shape[1]
    PS = kv_pages.shape[3]
    assert int(extend_lens.sum()) == T and k_new.shape == v_new.shape == (T, Hkv, D)
    assert kv_pages.shape[1:] == (2, Hkv, PS, D) and block_table.shape[0] == B
    if rows is None:
        n_rows, rp = T, None
    else:
        rows, rp = _i32(rows)
        n_rows = rows.shape[0]
        assert n_rows == 0 or (rows.min() >= 0 and rows.max() < T)
    out = np.zeros((n_rows, Hq, D), dtype=np.float64)
    lse = np.zeros((n_rows, Hq), dtype=np.float64)
    rc = lib.oracle_extend_attention(
        qp, kp, vp, pp, tp, plp, elp, B, Hq, Hkv, D, PS, block_table.shape[1],
        float(softmax_scale), rp, n_rows, int(key_lo), int(key_hi),
        out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
        lse.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise ValueError("oracle_extend_attention rejected its arguments")
    return (out, lse) if return_lse else out


def write_kv(k_new, v_new, kv_pages, block_table, prefix_lens, extend_lens) -> np.ndarray:
    """Returns a copy of kv_pages with the new K/V rows appended behind each prefix."""
    lib = _load()
    k_new, kp = _u16(k_new)
    v_new, vp = _u16(v_new)
    pool = np.array(kv_pages, dtype=np.uint16, order="C", copy=True)
    block_table, tp = _i32(block_table)
    prefix_lens, plp = _i32(prefix_lens)
    extend_lens, elp = _i32(extend_lens)
    T, Hkv, D = k_new.shape
    PS = pool.shape[3]
    assert int(extend_lens.sum()) == T and pool.shape[1:] == (2, Hkv, PS, D)
    rc = lib.oracle_write_kv(kp, vp, pool.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), tp,
                             plp, elp, prefix_lens.shape[0], Hkv, D, PS, block_table.shape[1])
    if rc != 0:
        raise ValueError("oracle_write_kv rejected its arguments")
    return pool


def attention_of(w, rows=None, **kw):
    """Oracle attention on a workloads.Workload-shaped object (duck-typed fields)."""
    return extend_attention(w.q, w.k_new, w.v_new, w.kv_pages, w.block_table, w.prefix_lens,
                            w.extend_lens, w.softmax_scale, rows=rows, **kw)


def context_distance(contexts, lens, alpha: float) -> np.ndarray:
    """Pairwise context distance (paper, Eq. 1) in fp64.

    contexts [n, stride] int32 (row i holds lens[i] distinct block ids in rank order),
    lens [n] int32.  Returns dist [n, n] float64.
    """
    lib = _load()
    contexts, cp_ = _i32(contexts)
    lens, lp = _i32(lens)
    n, stride = contexts.shape
    assert lens.shape == (n,)
    out = np.zeros((n, n), dtype=np.float64)
    rc = lib.oracle_context_distance(cp_, lp, n, stride, float(alpha),
                                     out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise ValueError("oracle_context_distance rejected its arguments")
    return out
