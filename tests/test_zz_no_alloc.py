"""cp_extend_attention_noalloc (scratch inside the library) against cp_extend_attention (caller's
workspace): same kernels, same plan, so the outputs must agree bit for bit.  Two calls in a row
share the library's array, the second with a smaller input."""
import numpy as np
import pytest
import torch

import paper_2511_03475_amd as cp
import workloads as W
from gpu_harness import DeviceCase

pytestmark = pytest.mark.gpu


def _both(w, num_splits=0):
    c = DeviceCase(w, num_splits)
    assert c.ws_bytes > 0, "the case must use scratch"
    c.out.fill_(0x7FC1)
    c.attention()
    want = c.out_bits().copy()
    c.out.fill_(0x7FC1)
    cp.cp_extend_attention_noalloc(c.q, c.k_new, c.v_new, c.kv_pages, c.block_table, c.prefix_lens,
                                   c.extend_lens, c.out, torch.cuda.current_stream(), c.shape)
    got = c.out_bits().copy()
    return got, want


def test_two_calls_in_a_row_the_second_smaller():
    # split-K of the row-tiled kernel (forced 3-way), then a smaller decode-shaped batch
    big = W.make_uniform("noalloc_big", 777, 3, 8, 2, [700, 33, 1500], [300, 129, 64])
    got, want = _both(big, num_splits=3)
    assert (got == want).all()
    small = W.make_uniform("noalloc_small", 778, 5, 8, 2, [260, 0, 1000, 17, 512], [1, 2, 1, 3, 1])
    got, want = _both(small)
    assert cp.cp_num_splits(DeviceCase(small).shape) >= 4      # the decode-shaped plan: partials + merge
    assert (got == want).all()
    # and the first shape again: stale partials of the smaller call must not leak in
    got, want = _both(big, num_splits=3)
    assert (got == want).all()


def test_unsplit_shapes_need_no_scratch_and_still_run():
    w = W.make_uniform("noalloc_unsplit", 779, 2, 8, 2, [100, 40], [300, 280])
    c = DeviceCase(w, 1)
    c.attention()
    want = c.out_bits().copy()
    c.out.fill_(0)
    cp.cp_extend_attention_noalloc(c.q, c.k_new, c.v_new, c.kv_pages, c.block_table, c.prefix_lens,
                                   c.extend_lens, c.out, torch.cuda.current_stream(), c.shape)
    assert (c.out_bits() == want).all()


def test_a_shape_beyond_the_scratch_size_is_refused_and_nothing_runs():
    limit = cp.cp_noalloc_scratch_bytes()
    assert limit == 64 << 20
    # 64 forced splits x 2048 rows x 8 heads x 130 floats = 545 MB of partials
    w = W.make_uniform("noalloc_too_big", 780, 1, 8, 2, 4096, 2048)
    c = DeviceCase(w, 64)
    assert c.ws_bytes > limit
    c.out.fill_(0x1234)
    st = cp.cp_extend_attention_noalloc(c.q, c.k_new, c.v_new, c.kv_pages, c.block_table, c.prefix_lens,
                                        c.extend_lens, c.out, torch.cuda.current_stream(), c.shape, check=False)
    assert st == cp.CP_ERR_WORKSPACE
    assert (c.out_bits() == 0x1234).all()


def test_the_call_can_be_recorded_into_a_hip_graph_and_replayed():
    """What the entry point is for: under stream capture nothing may allocate.  The call is made
    once eagerly (the scratch address of the device is looked up then), recorded into a graph and
    replayed three times with eager work in between; every replay must reproduce the eager bits."""
    w = W.make_uniform("noalloc_graph", 781, 4, 8, 2, [900, 0, 2500, 64], [1, 3, 2, 1])    # decode-shaped: partials + merge
    c = DeviceCase(w)
    assert c.ws_bytes > 0
    s = torch.cuda.current_stream()
    call = lambda stream: cp.cp_extend_attention_noalloc(c.q, c.k_new, c.v_new, c.kv_pages, c.block_table,
                                                         c.prefix_lens, c.extend_lens, c.out, stream, c.shape)
    call(s)
    want = c.out_bits().copy()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(torch.cuda.current_stream())
    other = DeviceCase(W.make_uniform("noalloc_other", 782, 2, 8, 2, [300, 40], [200, 90]), 3)
    for _ in range(3):
        c.out.fill_(0x7FC1)
        other.attention()                       # eager work that uses the same scratch in between
        cp.cp_extend_attention_noalloc(other.q, other.k_new, other.v_new, other.kv_pages, other.block_table,
                                       other.prefix_lens, other.extend_lens, other.out, s, other.shape)
        torch.cuda.synchronize()
        graph.replay()
        assert (c.out_bits() == want).all()
