"""ctypes binding of libcp_extend.so: argument marshalling only.

Every function has the name and argument order of its C entry point (include/cp_extend.h).
Device buffers are anything with a ``data_ptr()`` method (torch tensors) or raw integer
addresses; nothing is computed here and there is no fallback: if the library has not been
built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

from .build import LIB_PATH

CP_OK = 0
CP_ERR_NULL = -1
CP_ERR_SHAPE = -2
CP_ERR_WORKSPACE = -3
CP_ERR_LAUNCH = -4

EXPORTS = ("cp_workspace_bytes", "cp_num_splits", "cp_extend_attention", "cp_write_kv",
           "cp_status_string", "cp_context_distance", "cp_probe_mfma",
           "cp_probe_mfma_sink_floats", "cp_probe_mfma_flops")


class cp_shape(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("num_pages", ctypes.c_int32),
        ("max_pages_per_req", ctypes.c_int32), ("total_extend", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float), ("num_splits", ctypes.c_int32),
        ("h_prefix_lens", ctypes.POINTER(ctypes.c_int32)),
        ("h_extend_lens", ctypes.POINTER(ctypes.c_int32)),
    ]


class CpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {cp_status_string(status)} (status {status})")


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    # PyTorch ships its own copy of the HIP runtime; if this library were loaded first it
    # would bring in the system copy, and the two runtimes do not share devices or streams.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it first (python -m paper_2511_03475_amd.build)")
    lib = ctypes.CDLL(path)
    vp, i32p, sp = ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(cp_shape)
    lib.cp_workspace_bytes.restype = ctypes.c_size_t
    lib.cp_workspace_bytes.argtypes = [sp]
    lib.cp_num_splits.restype = ctypes.c_int32
    lib.cp_num_splits.argtypes = [sp]
    lib.cp_extend_attention.restype = ctypes.c_int
    lib.cp_extend_attention.argtypes = [vp, vp, vp, vp, i32p, i32p, i32p, vp, vp, sp, vp, ctypes.c_size_t]
    lib.cp_write_kv.restype = ctypes.c_int
    lib.cp_write_kv.argtypes = [vp, vp, vp, i32p, i32p, i32p, vp, sp]
    lib.cp_context_distance.restype = ctypes.c_int
    lib.cp_context_distance.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_float, vp, vp]
    lib.cp_probe_mfma.restype = ctypes.c_int
    lib.cp_probe_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, vp]
    lib.cp_probe_mfma_sink_floats.restype = ctypes.c_size_t
    lib.cp_probe_mfma_sink_floats.argtypes = []
    lib.cp_probe_mfma_flops.restype = ctypes.c_double
    lib.cp_probe_mfma_flops.argtypes = [ctypes.c_int32]
    lib.cp_status_string.restype = ctypes.c_char_p
    lib.cp_status_string.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x or None
    return int(x.data_ptr()) or None


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


class Shape:
    """Owns a cp_shape and the host length arrays it points to."""

    def __init__(self, batch: int, num_q_heads: int, num_kv_heads: int, head_dim: int,
                 page_size: int, num_pages: int, max_pages_per_req: int,
                 prefix_lens: Sequence[int], extend_lens: Sequence[int], softmax_scale: float,
                 num_splits: int = 0, total_extend: Optional[int] = None):
        self._p = np.ascontiguousarray(prefix_lens, dtype=np.int32)
        self._e = np.ascontiguousarray(extend_lens, dtype=np.int32)
        if total_extend is None:
            total_extend = int(self._e.astype(np.int64).sum())
        i32p = ctypes.POINTER(ctypes.c_int32)
        self.c = cp_shape(batch, num_q_heads, num_kv_heads, head_dim, page_size, num_pages,
                          max_pages_per_req, total_extend, softmax_scale, num_splits,
                          self._p.ctypes.data_as(i32p), self._e.ctypes.data_as(i32p))

    def ref(self):
        return ctypes.byref(self.c)


def cp_status_string(status: int) -> str:
    return load_library().cp_status_string(int(status)).decode()


def cp_workspace_bytes(shape: Shape) -> int:
    return int(load_library().cp_workspace_bytes(shape.ref()))


def cp_num_splits(shape: Shape) -> int:
    return int(load_library().cp_num_splits(shape.ref()))


def cp_extend_attention(q, k_new, v_new, kv_pages, block_table, prefix_lens, extend_lens, out,
                        stream, shape: Shape, workspace=None, workspace_bytes: int = 0,
                        check: bool = True) -> int:
    st = load_library().cp_extend_attention(
        _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kv_pages), _ptr(block_table), _ptr(prefix_lens),
        _ptr(extend_lens), _ptr(out), _stream(stream), shape.ref(), _ptr(workspace),
        int(workspace_bytes))
    if check and st != CP_OK:
        raise CpError(st, "cp_extend_attention")
    return st


def cp_write_kv(k_new, v_new, kv_pages, block_table, prefix_lens, extend_lens, stream,
                shape: Shape, check: bool = True) -> int:
    st = load_library().cp_write_kv(
        _ptr(k_new), _ptr(v_new), _ptr(kv_pages), _ptr(block_table), _ptr(prefix_lens),
        _ptr(extend_lens), _stream(stream), shape.ref())
    if check and st != CP_OK:
        raise CpError(st, "cp_write_kv")
    return st


def cp_context_distance(contexts, lens, n: int, stride: int, alpha: float, dist, stream,
                        check: bool = True) -> int:
    st = load_library().cp_context_distance(_ptr(contexts), _ptr(lens), int(n), int(stride),
                                            float(alpha), _ptr(dist), _stream(stream))
    if check and st != CP_OK:
        raise CpError(st, "cp_context_distance")
    return st


def cp_probe_mfma(random_operands: bool, iters: int, sink, stream, check: bool = True) -> int:
    st = load_library().cp_probe_mfma(int(bool(random_operands)), int(iters), _ptr(sink), _stream(stream))
    if check and st != CP_OK:
        raise CpError(st, "cp_probe_mfma")
    return st


def cp_probe_mfma_sink_floats() -> int:
    return int(load_library().cp_probe_mfma_sink_floats())


def cp_probe_mfma_flops(iters: int) -> float:
    return float(load_library().cp_probe_mfma_flops(int(iters)))
