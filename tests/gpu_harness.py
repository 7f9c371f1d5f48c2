"""Runs the HIP library on a workloads.Workload: device buffers via torch, calls via the C ABI."""
import numpy as np
import torch

import paper_2511_03475_amd as cp


def _dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).to("cuda:0", non_blocking=False)


class DeviceCase:
    """Device-resident copy of a workload plus the cp_shape describing it."""

    def __init__(self, w, num_splits: int = 0):
        self.w = w
        self.q = _dev(w.q)
        self.k_new = _dev(w.k_new)
        self.v_new = _dev(w.v_new)
        self.kv_pages = _dev(w.kv_pages)
        self.block_table = _dev(w.block_table)
        self.prefix_lens = _dev(w.prefix_lens)
        self.extend_lens = _dev(w.extend_lens)
        self.out = torch.empty((max(w.total_extend, 1), w.num_q_heads, w.head_dim),
                               dtype=torch.int16, device="cuda:0")
        self.set_splits(num_splits)

    def set_splits(self, num_splits: int):
        w = self.w
        self.shape = cp.Shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.page_size,
                              w.num_pages, w.max_pages_per_req, w.prefix_lens, w.extend_lens,
                              w.softmax_scale, num_splits=num_splits)
        self.ws_bytes = cp.cp_workspace_bytes(self.shape)
        self.workspace = (torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda:0")
                          if self.ws_bytes else None)

    def attention(self, stream=None):
        s = stream if stream is not None else torch.cuda.current_stream()
        cp.cp_extend_attention(self.q, self.k_new, self.v_new, self.kv_pages, self.block_table,
                               self.prefix_lens, self.extend_lens, self.out, s, self.shape,
                               self.workspace, self.ws_bytes)

    def write_kv(self, stream=None):
        s = stream if stream is not None else torch.cuda.current_stream()
        cp.cp_write_kv(self.k_new, self.v_new, self.kv_pages, self.block_table,
                       self.prefix_lens, self.extend_lens, s, self.shape)

    def out_bits(self) -> np.ndarray:
        torch.cuda.synchronize()
        T = self.w.total_extend
        return self.out[:T].cpu().numpy().view(np.uint16)

    def pool_bits(self) -> np.ndarray:
        torch.cuda.synchronize()
        return self.kv_pages.cpu().numpy().view(np.uint16)


def gpu_attention(w, num_splits: int = 0) -> np.ndarray:
    """bf16 bit patterns [T, Hq, D] computed by cp_extend_attention."""
    case = DeviceCase(w, num_splits)
    case.attention()
    return case.out_bits()
