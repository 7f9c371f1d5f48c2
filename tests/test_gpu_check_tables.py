"""cp_check_tables and debug mode: a block table with a page id outside the pool, or device
lengths that differ from the host copies, are reported as errors and nothing is launched on them.
The bad tables here are only ever read by the checking kernel, which follows no page id."""
import numpy as np
import pytest
import torch

import paper_2511_03475_amd as cp
import workloads as W
from gpu_harness import DeviceCase

pytestmark = pytest.mark.gpu


@pytest.fixture()
def case():
    w = W.make_uniform("check", 4242, 3, 8, 2, 300, 40)   # 3 requests, 22 pages each (the last partly filled)
    return DeviceCase(w)


def _check(c):
    return cp.cp_check_tables(c.block_table, c.prefix_lens, c.extend_lens, torch.cuda.current_stream(),
                              c.shape, check=False)


def test_a_consistent_batch_passes(case):
    st, info = _check(case)
    assert st == cp.CP_OK and info == [-1, -1, -1]


@pytest.mark.parametrize("bad", [-1, -7, None])           # None: num_pages itself, the first id past the pool
def test_a_page_id_outside_the_pool_is_reported_with_its_place(case, bad):
    w = case.w
    value = w.num_pages if bad is None else bad
    used = (300 + 40 + 15) // 16
    table = w.block_table.copy()
    table[2, used - 1] = value + 5                         # a later offence: the first one is reported
    table[1, 7] = value
    case.block_table = torch.from_numpy(table).to("cuda:0")
    st, info = _check(case)
    assert st == cp.CP_ERR_TABLE and info == [1, 7, value]


def test_entries_beyond_the_pages_in_use_are_ignored(case):
    w = case.w
    used = (300 + 40 + 15) // 16
    assert w.block_table.shape[1] >= used
    table = np.concatenate([w.block_table, np.full((3, 5), -1, np.int32)], axis=1)
    sh = cp.Shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.page_size, w.num_pages, table.shape[1],
                  w.prefix_lens, w.extend_lens, w.softmax_scale)
    st, _ = cp.cp_check_tables(torch.from_numpy(table).to("cuda:0"), case.prefix_lens, case.extend_lens,
                               torch.cuda.current_stream(), sh, check=False)
    assert st == cp.CP_OK


def test_device_lengths_that_differ_from_the_host_copies_are_reported(case):
    pl = case.w.prefix_lens.copy()
    pl[1] += 16
    case.prefix_lens = torch.from_numpy(pl).to("cuda:0")
    st, info = _check(case)
    assert st == cp.CP_ERR_LENGTHS and info == [1, int(pl[1]), int(case.w.extend_lens[1])]


def test_debug_mode_refuses_to_launch_on_a_bad_table(case):
    """With debug mode on, both entry points run the check first; the output buffer and the
    page pool keep their sentinel, so no kernel ran on the bad table."""
    w = case.w
    table = w.block_table.copy()
    table[0, 3] = w.num_pages + 1000
    case.block_table = torch.from_numpy(table).to("cuda:0")
    case.out.fill_(0x1234)
    pool_before = case.pool_bits().copy()
    s = torch.cuda.current_stream()
    cp.cp_set_debug_validate(True)
    try:
        st_a = cp.cp_extend_attention(case.q, case.k_new, case.v_new, case.kv_pages, case.block_table,
                                      case.prefix_lens, case.extend_lens, case.out, s, case.shape, case.workspace,
                                      case.ws_bytes, check=False)
        st_w = cp.cp_write_kv(case.k_new, case.v_new, case.kv_pages, case.block_table, case.prefix_lens,
                              case.extend_lens, s, case.shape, check=False)
        # a good table still runs in debug mode, and gives what it gives without it
        good = DeviceCase(w)
        good.attention()
        with_debug = good.out_bits().copy()
    finally:
        cp.cp_set_debug_validate(False)
    assert st_a == cp.CP_ERR_TABLE and st_w == cp.CP_ERR_TABLE
    assert (case.out_bits() == 0x1234).all()
    assert (case.pool_bits() == pool_before).all()
    good.attention()
    assert (good.out_bits() == with_debug).all()


def test_batches_beyond_one_grid_dimension_are_checked_in_full():
    """70000 one-token requests: the check walks the batch in pieces of 65535 requests; an offence in
    the second piece is found and reported with its request number."""
    B = 70000
    table = np.arange(B, dtype=np.int32).reshape(B, 1)
    zeros, ones = np.zeros(B, np.int32), np.ones(B, np.int32)
    sh = cp.Shape(B, 2, 1, 128, 16, B, 1, zeros, ones, 0.1)
    dev = lambda a: torch.from_numpy(a).to("cuda:0")
    s = torch.cuda.current_stream()
    st, info = cp.cp_check_tables(dev(table), dev(zeros), dev(ones), s, sh, check=False)
    assert st == cp.CP_OK
    table[66000, 0] = B
    st, info = cp.cp_check_tables(dev(table), dev(zeros), dev(ones), s, sh, check=False)
    assert st == cp.CP_ERR_TABLE and info == [66000, 0, B]
    table[123, 0] = -5
    st, info = cp.cp_check_tables(dev(table), dev(zeros), dev(ones), s, sh, check=False)
    assert st == cp.CP_ERR_TABLE and info == [123, 0, -5]
