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
CP_ERR_ALIGN = -5
CP_ERR_TABLE = -6
CP_ERR_LENGTHS = -7

EXPORTS = ("cp_workspace_bytes", "cp_num_splits", "cp_plan_kind", "cp_extend_attention", "cp_write_kv",
           "cp_extend_attention_noalloc", "cp_noalloc_scratch_bytes",
           "cp_status_string", "cp_check_tables", "cp_set_debug_validate", "cp_context_distance", "cp_probe_mfma", "cp_probe_mix", "cp_probe_copy", "cp_probe_fill_lds",
           "cp_probe_mfma_sink_floats", "cp_probe_mfma_flops",
           "cp_index_distinct", "cp_index_build", "cp_index_free", "cp_index_num_contexts",
           "cp_index_num_nodes", "cp_index_aligned", "cp_index_path", "cp_index_leaf", "cp_index_node",
           "cp_index_children", "cp_index_search", "cp_index_insert", "cp_index_schedule",
           "cp_dedup_hash", "cp_dedup_chunks", "cp_dedup_create", "cp_dedup_free", "cp_dedup_turn")


class cp_dedup_sub(ctypes.Structure):
    _fields_ = [("block", ctypes.c_int32), ("ref", ctypes.c_int32), ("begin", ctypes.c_int64),
                ("end", ctypes.c_int64)]


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
    lib.cp_plan_kind.restype = ctypes.c_int32
    lib.cp_plan_kind.argtypes = [sp]
    lib.cp_extend_attention.restype = ctypes.c_int
    lib.cp_extend_attention.argtypes = [vp, vp, vp, vp, i32p, i32p, i32p, vp, vp, sp, vp, ctypes.c_size_t]
    lib.cp_extend_attention_noalloc.restype = ctypes.c_int
    lib.cp_extend_attention_noalloc.argtypes = [vp, vp, vp, vp, i32p, i32p, i32p, vp, vp, sp]
    lib.cp_noalloc_scratch_bytes.restype = ctypes.c_size_t
    lib.cp_noalloc_scratch_bytes.argtypes = []
    lib.cp_write_kv.restype = ctypes.c_int
    lib.cp_write_kv.argtypes = [vp, vp, vp, i32p, i32p, i32p, vp, sp]
    lib.cp_check_tables.restype = ctypes.c_int
    lib.cp_check_tables.argtypes = [i32p, i32p, i32p, vp, sp, ctypes.POINTER(ctypes.c_int32)]
    lib.cp_set_debug_validate.restype = None
    lib.cp_set_debug_validate.argtypes = [ctypes.c_int]
    lib.cp_context_distance.restype = ctypes.c_int
    lib.cp_context_distance.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_float, vp, vp]
    lib.cp_probe_mfma.restype = ctypes.c_int
    lib.cp_probe_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, vp]
    lib.cp_probe_mix.restype = ctypes.c_int
    lib.cp_probe_mix.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, vp]
    lib.cp_probe_copy.restype = ctypes.c_int
    lib.cp_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.cp_probe_fill_lds.restype = ctypes.c_int
    lib.cp_probe_fill_lds.argtypes = [ctypes.c_uint32, vp]
    lib.cp_probe_mfma_sink_floats.restype = ctypes.c_size_t
    lib.cp_probe_mfma_sink_floats.argtypes = []
    lib.cp_probe_mfma_flops.restype = ctypes.c_double
    lib.cp_probe_mfma_flops.argtypes = [ctypes.c_int32]
    i32, i32p, f64p = ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)
    lib.cp_index_distinct.restype = ctypes.c_int
    lib.cp_index_distinct.argtypes = [i32p, i32p, i32, i32, i32p, i32p]
    lib.cp_index_build.restype = ctypes.c_int
    lib.cp_index_build.argtypes = [i32p, i32p, i32, i32, ctypes.c_double, ctypes.POINTER(ctypes.c_float), i32,
                                   ctypes.POINTER(vp)]
    lib.cp_index_free.restype = None
    lib.cp_index_free.argtypes = [vp]
    lib.cp_index_num_contexts.restype = i32
    lib.cp_index_num_contexts.argtypes = [vp]
    lib.cp_index_num_nodes.restype = i32
    lib.cp_index_num_nodes.argtypes = [vp]
    lib.cp_index_aligned.restype = ctypes.c_int
    lib.cp_index_aligned.argtypes = [vp, i32, i32p, i32, i32p]
    lib.cp_index_path.restype = ctypes.c_int
    lib.cp_index_path.argtypes = [vp, i32, i32p, i32, i32p]
    lib.cp_index_leaf.restype = ctypes.c_int
    lib.cp_index_leaf.argtypes = [vp, i32, i32p]
    lib.cp_index_node.restype = ctypes.c_int
    lib.cp_index_node.argtypes = [vp, i32, i32p, i32p, i32p, f64p, i32p, i32p, i32, i32p]
    lib.cp_index_children.restype = ctypes.c_int
    lib.cp_index_children.argtypes = [vp, i32, i32p, i32, i32p]
    lib.cp_index_search.restype = ctypes.c_int
    lib.cp_index_search.argtypes = [vp, i32p, i32, i32p, i32, i32p, i32p]
    lib.cp_index_insert.restype = ctypes.c_int
    lib.cp_index_insert.argtypes = [vp, i32p, i32, i32p, i32p, i32, i32p]
    lib.cp_index_schedule.restype = ctypes.c_int
    lib.cp_index_schedule.argtypes = [i32p, i32p, i32, i32, i32p]
    u8p, i64p = ctypes.POINTER(ctypes.c_uint8), ctypes.POINTER(ctypes.c_int64)
    lib.cp_dedup_hash.restype = ctypes.c_uint64
    lib.cp_dedup_hash.argtypes = [u8p, ctypes.c_int64]
    lib.cp_dedup_chunks.restype = ctypes.c_int
    lib.cp_dedup_chunks.argtypes = [u8p, ctypes.c_int64, ctypes.c_uint64, i64p, i32, i32p]
    lib.cp_dedup_create.restype = ctypes.c_int
    lib.cp_dedup_create.argtypes = [ctypes.c_uint64, ctypes.POINTER(vp)]
    lib.cp_dedup_free.restype = None
    lib.cp_dedup_free.argtypes = [vp]
    lib.cp_dedup_turn.restype = ctypes.c_int
    lib.cp_dedup_turn.argtypes = [vp, i32p, u8p, i64p, i32, i32p, ctypes.POINTER(cp_dedup_sub), i32, i32p, i64p]
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


PLAN_KERNELS = {1: "extend_attn_kernel", 2: "extend_attn_kernel + merge_splits_kernel",
                3: "decode_attn_kernel + merge_splits_kernel"}


def cp_plan_kind(shape: Shape) -> int:
    return int(load_library().cp_plan_kind(shape.ref()))


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


def cp_extend_attention_noalloc(q, k_new, v_new, kv_pages, block_table, prefix_lens, extend_lens, out,
                                stream, shape: Shape, check: bool = True) -> int:
    st = load_library().cp_extend_attention_noalloc(
        _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kv_pages), _ptr(block_table), _ptr(prefix_lens),
        _ptr(extend_lens), _ptr(out), _stream(stream), shape.ref())
    if check and st != CP_OK:
        raise CpError(st, "cp_extend_attention_noalloc")
    return st


def cp_noalloc_scratch_bytes() -> int:
    return int(load_library().cp_noalloc_scratch_bytes())


def cp_write_kv(k_new, v_new, kv_pages, block_table, prefix_lens, extend_lens, stream,
                shape: Shape, check: bool = True) -> int:
    st = load_library().cp_write_kv(
        _ptr(k_new), _ptr(v_new), _ptr(kv_pages), _ptr(block_table), _ptr(prefix_lens),
        _ptr(extend_lens), _stream(stream), shape.ref())
    if check and st != CP_OK:
        raise CpError(st, "cp_write_kv")
    return st


def cp_check_tables(block_table, prefix_lens, extend_lens, stream, shape: Shape, check: bool = True):
    """(status, [a, b, c]): see the header for the meaning of the three numbers."""
    info = (ctypes.c_int32 * 3)(-1, -1, -1)
    st = load_library().cp_check_tables(_ptr(block_table), _ptr(prefix_lens), _ptr(extend_lens),
                                        _stream(stream), shape.ref(), info)
    if check and st != CP_OK:
        raise CpError(st, "cp_check_tables")
    return st, [int(x) for x in info]


def cp_set_debug_validate(on: bool) -> None:
    load_library().cp_set_debug_validate(int(bool(on)))


def cp_context_distance(contexts, lens, n: int, stride: int, alpha: float, dist, stream,
                        check: bool = True) -> int:
    st = load_library().cp_context_distance(_ptr(contexts), _ptr(lens), int(n), int(stride),
                                            float(alpha), _ptr(dist), _stream(stream))
    if check and st != CP_OK:
        raise CpError(st, "cp_context_distance")
    return st


def cp_probe_mfma(operands: int, iters: int, sink, stream, check: bool = True) -> int:
    st = load_library().cp_probe_mfma(int(operands), int(iters), _ptr(sink), _stream(stream))
    if check and st != CP_OK:
        raise CpError(st, "cp_probe_mfma")
    return st


def cp_probe_mix(operands: int, iters: int, sink, stream, check: bool = True) -> int:
    st = load_library().cp_probe_mix(int(operands), int(iters), _ptr(sink), _stream(stream))
    if check and st != CP_OK:
        raise CpError(st, "cp_probe_mix")
    return st


def cp_probe_fill_lds(pattern: int, stream, check: bool = True) -> int:
    """Fills the LDS of every compute unit with a 32-bit pattern (test aid, see cp_probe.h)."""
    st = load_library().cp_probe_fill_lds(int(pattern) & 0xFFFFFFFF, _stream(stream))
    if check and st != 0:
        raise CpError(st, "cp_probe_fill_lds")
    return st


def cp_probe_copy(dst, src, nbytes: int, stream, check: bool = True) -> int:
    st = load_library().cp_probe_copy(_ptr(dst), _ptr(src), int(nbytes), _stream(stream))
    if check and st != CP_OK:
        raise CpError(st, "cp_probe_copy")
    return st


def cp_probe_mfma_sink_floats() -> int:
    return int(load_library().cp_probe_mfma_sink_floats())


def cp_probe_mfma_flops(iters: int) -> float:
    return float(load_library().cp_probe_mfma_flops(int(iters)))


# ---- context index (host memory only; numpy arrays in, numpy arrays / lists out) -------------
def _i32_array(a):
    import numpy as np
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _check_index(st: int, what: str) -> None:
    if st != CP_OK:
        raise CpError(st, what)


def cp_index_distinct(contexts, lens):
    """first_of [n] int32 and the number of distinct contexts."""
    import numpy as np
    contexts, cptr = _i32_array(contexts)
    lens, lptr = _i32_array(lens)
    n, stride = contexts.shape
    first_of = np.zeros(n, dtype=np.int32)
    m = ctypes.c_int32(0)
    _check_index(load_library().cp_index_distinct(cptr, lptr, n, stride,
                                                  first_of.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                                  ctypes.byref(m)), "cp_index_distinct")
    return first_of, int(m.value)


class ContextIndex:
    """Owner of a cp_index handle.  Every method is one C call plus argument marshalling."""

    PATH_CAP = 4096

    def __init__(self, contexts, lens, alpha: float, dist=None):
        import numpy as np
        contexts, cptr = _i32_array(contexts)
        lens, lptr = _i32_array(lens)
        n, stride = contexts.shape
        dptr, m = None, 0
        if dist is not None:
            dist = np.ascontiguousarray(dist, dtype=np.float32)
            m = dist.shape[0]
            dptr = dist.ctypes.data_as(ctypes.POINTER(ctypes.c_float))
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        _check_index(self._lib.cp_index_build(cptr, lptr, n, stride, float(alpha), dptr, m,
                                              ctypes.byref(self._h)), "cp_index_build")

    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.cp_index_free(self._h)
            self._h = ctypes.c_void_p()

    __del__ = close

    def num_contexts(self) -> int:
        return int(self._lib.cp_index_num_contexts(self._h))

    def num_nodes(self) -> int:
        return int(self._lib.cp_index_num_nodes(self._h))

    def _list(self, fn, what, *args):
        buf = (ctypes.c_int32 * self.PATH_CAP)()
        n = ctypes.c_int32(0)
        _check_index(fn(self._h, *args, buf, self.PATH_CAP, ctypes.byref(n)), what)
        return [int(buf[i]) for i in range(n.value)]

    def aligned(self, i: int):
        return self._list(self._lib.cp_index_aligned, "cp_index_aligned", int(i))

    def path(self, i: int):
        return self._list(self._lib.cp_index_path, "cp_index_path", int(i))

    def leaf(self, i: int) -> int:
        node = ctypes.c_int32(0)
        _check_index(self._lib.cp_index_leaf(self._h, int(i), ctypes.byref(node)), "cp_index_leaf")
        return int(node.value)

    def children(self, node: int):
        return self._list(self._lib.cp_index_children, "cp_index_children", int(node))

    def node(self, node: int) -> dict:
        parent, leaf, freq, nch, n = (ctypes.c_int32(0) for _ in range(5))
        created = ctypes.c_double(0.0)
        buf = (ctypes.c_int32 * self.PATH_CAP)()
        _check_index(self._lib.cp_index_node(self._h, int(node), ctypes.byref(parent), ctypes.byref(leaf),
                                             ctypes.byref(freq), ctypes.byref(created), ctypes.byref(nch), buf,
                                             self.PATH_CAP, ctypes.byref(n)), "cp_index_node")
        return {"parent": int(parent.value), "leaf": bool(leaf.value), "freq": int(freq.value),
                "created_at": float(created.value), "num_children": int(nch.value),
                "docs": [int(buf[i]) for i in range(n.value)]}

    def search(self, ids):
        ids, iptr = _i32_array(ids)
        buf = (ctypes.c_int32 * self.PATH_CAP)()
        n, node = ctypes.c_int32(0), ctypes.c_int32(0)
        _check_index(self._lib.cp_index_search(self._h, iptr, len(ids), buf, self.PATH_CAP, ctypes.byref(n),
                                               ctypes.byref(node)), "cp_index_search")
        return [int(buf[i]) for i in range(n.value)], int(node.value)

    def insert(self, ids):
        import numpy as np
        ids, iptr = _i32_array(ids)
        aligned = np.zeros(max(len(ids), 1), dtype=np.int32)
        buf = (ctypes.c_int32 * self.PATH_CAP)()
        n = ctypes.c_int32(0)
        _check_index(self._lib.cp_index_insert(self._h, iptr, len(ids),
                                               aligned.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), buf,
                                               self.PATH_CAP, ctypes.byref(n)), "cp_index_insert")
        return [int(x) for x in aligned[:len(ids)]], [int(buf[i]) for i in range(n.value)]


def cp_index_schedule(paths):
    """Execution order (list of indices) for a list of search paths."""
    import numpy as np
    n = len(paths)
    stride = max([len(p) for p in paths] + [1])
    P = np.zeros((max(n, 1), stride), dtype=np.int32)
    L = np.zeros(max(n, 1), dtype=np.int32)
    for i, p in enumerate(paths):
        P[i, :len(p)] = p
        L[i] = len(p)
    order = np.zeros(max(n, 1), dtype=np.int32)
    _check_index(load_library().cp_index_schedule(P.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                                  L.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), n, stride,
                                                  order.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))),
                 "cp_index_schedule")
    return [int(x) for x in order[:n]]


# ---- context de-duplication (host memory only) -----------------------------------------------
def _u8(data: bytes):
    buf = (ctypes.c_uint8 * max(len(data), 1)).from_buffer_copy(data if data else b"\0")
    return buf


def cp_dedup_hash(data: bytes) -> int:
    return int(load_library().cp_dedup_hash(_u8(data), len(data)))


def cp_dedup_chunks(data: bytes, modulus: int):
    """End offsets of the sub-blocks of one block."""
    cap = data.count(b"\n") + 2
    ends = (ctypes.c_int64 * cap)()
    n = ctypes.c_int32(0)
    _check_index(load_library().cp_dedup_chunks(_u8(data), len(data), int(modulus), ends, cap, ctypes.byref(n)),
                 "cp_dedup_chunks")
    return [int(ends[i]) for i in range(n.value)]


class Conversation:
    """Owner of a cp_dedup handle.  turn() is one C call plus argument marshalling."""

    def __init__(self, modulus: int):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        _check_index(self._lib.cp_dedup_create(int(modulus), ctypes.byref(self._h)), "cp_dedup_create")

    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.cp_dedup_free(self._h)
            self._h = ctypes.c_void_p()

    __del__ = close

    def turn(self, ids, blocks):
        """Per block ("block", id) or ("subs", [(begin, end, ref), ...]), and the kept bytes."""
        n = len(ids)
        data = b"".join(blocks)
        offsets = (ctypes.c_int64 * (n + 1))()
        at = 0
        for i, b in enumerate(blocks):
            offsets[i] = at
            at += len(b)
        offsets[n] = at
        idv = (ctypes.c_int32 * max(n, 1))(*[int(i) for i in ids])
        ref = (ctypes.c_int32 * max(n, 1))()
        cap = data.count(b"\n") + n + 1
        subs = (cp_dedup_sub * cap)()
        cnt, kept = ctypes.c_int32(0), ctypes.c_int64(0)
        _check_index(self._lib.cp_dedup_turn(self._h, idv, _u8(data), offsets, n, ref, subs, cap,
                                             ctypes.byref(cnt), ctypes.byref(kept)), "cp_dedup_turn")
        out = [("block", int(ids[i])) if ref[i] else ("subs", []) for i in range(n)]
        for k in range(cnt.value):
            s = subs[k]
            out[s.block][1].append((int(s.begin), int(s.end), int(s.ref)))
        return out, int(kept.value)
