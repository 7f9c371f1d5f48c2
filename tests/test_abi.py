"""The C-ABI library loads, exports every function the header declares, and its host-side
argument checks and launch planning work without a GPU (no kernel is launched here)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2511_03475_amd as cp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(cp.LIB_PATH):
        cp.build()
    return cp.load_library()


def _declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, f)).read(), flags=re.S)
            names |= set(re.findall(r"\b(cp_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert set(names) == set(cp.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    assert cp.cp_status_string(cp.CP_OK) == "ok"
    texts = [cp.cp_status_string(code) for code in (cp.CP_ERR_NULL, cp.CP_ERR_SHAPE, cp.CP_ERR_WORKSPACE,
                                                    cp.CP_ERR_LAUNCH, cp.CP_ERR_ALIGN, cp.CP_ERR_TABLE,
                                                    cp.CP_ERR_LENGTHS, -99)]
    assert all(len(t) > 3 for t in texts) and len(set(texts)) == len(texts)


def _shape(P, E, Hq=32, Hkv=8, splits=0, D=128, PS=16, pages=None, width=None):
    need = max((p + e + 15) // 16 for p, e in zip(P, E))
    return cp.Shape(len(P), Hq, Hkv, D, PS, pages or 100000, width or max(need, 1), P, E,
                    1.0 / np.sqrt(128), num_splits=splits)


def test_split_plan_is_a_pure_function_of_the_shape(lib):
    big = _shape([24576] * 4, [8192] * 4, Hq=64)
    assert cp.cp_num_splits(big) == 1 and cp.cp_workspace_bytes(big) == 0
    forced = _shape([24576] * 4, [8192] * 4, Hq=64, splits=2)
    assert cp.cp_num_splits(forced) == 2
    rows = 2 * 4 * 8192 * 64
    assert cp.cp_workspace_bytes(forced) == rows * 128 * 4 + rows * 2 * 4
    short = _shape([10240], [128])           # one short request: few workgroups -> split
    ns = cp.cp_num_splits(short)
    assert 1 < ns <= 64 and cp.cp_workspace_bytes(short) > 0
    assert cp.cp_num_splits(_shape([10240], [128])) == ns


def test_decode_shaped_calls_get_a_wavefront_level_plan(lib):
    """Few rows per (request, KV head): the library merges many wavefront-sized key chunks, a
    multiple of the four wavefronts of a workgroup; a forced split count keeps the row-tiled
    kernel."""
    dec = _shape([10240] * 32, [1] * 32)
    ns = cp.cp_num_splits(dec)
    assert ns >= 4 and ns % 4 == 0 and ns <= 256
    rows = ns * 32 * 32
    assert cp.cp_workspace_bytes(dec) == rows * 128 * 4 + rows * 2 * 4
    assert cp.cp_num_splits(_shape([10240] * 32, [1] * 32, splits=1)) == 1
    one = cp.cp_num_splits(_shape([131072], [1]))
    assert one % 4 == 0 and one > ns
    tiny = cp.cp_num_splits(_shape([0, 3], [2, 1]))          # at most 2 blocks of keys per chunk
    assert tiny == 4
    # G * E = 4 * 17 = 68 rows per KV head is past the decode-shaped limit
    assert cp.cp_num_splits(_shape([10240] * 64, [17] * 64)) == 1


def test_plan_kind_names_the_kernels_that_will_run(lib):
    assert cp.cp_plan_kind(_shape([24576] * 4, [8192] * 4, Hq=64)) == 1          # row-tiled, unsplit
    assert cp.cp_plan_kind(_shape([24576] * 4, [8192] * 4, Hq=64, splits=2)) == 2
    assert cp.cp_plan_kind(_shape([10240], [128])) == 2                           # few workgroups: split
    assert cp.cp_plan_kind(_shape([10240] * 32, [1] * 32)) == 3                   # decode-shaped
    assert cp.cp_plan_kind(_shape([10240] * 32, [1] * 32, splits=1)) == 1
    assert cp.cp_plan_kind(_shape([32], [32], D=64)) == 0
    assert set(cp.PLAN_KERNELS) == {1, 2, 3}


def test_invalid_shapes_are_rejected_on_the_host(lib):
    bad = [
        _shape([32], [32], Hq=4, Hkv=3),           # Hq % Hkv != 0
        _shape([32], [32], D=64),                  # head_dim
        _shape([32], [32], PS=32),                 # page_size
        _shape([32], [32], width=1),               # table too narrow
        _shape([-1], [32], width=4),               # negative length
        _shape([32], [32], splits=65),             # split factor out of range
    ]
    for sh in bad:
        assert cp.cp_num_splits(sh) == 0 and cp.cp_workspace_bytes(sh) == 0
        st = cp.cp_extend_attention(1, 1, 1, 1, 1, 1, 1, 1, None, sh, None, 0, check=False)
        assert st == cp.CP_ERR_SHAPE
        st = cp.cp_write_kv(1, 1, 1, 1, 1, 1, None, sh, check=False)
        assert st == cp.CP_ERR_SHAPE
    wrong_total = cp.Shape(1, 4, 2, 128, 16, 64, 8, [32], [32], 0.1, total_extend=31)
    assert cp.cp_extend_attention(1, 1, 1, 1, 1, 1, 1, 1, None, wrong_total, None, 0,
                                  check=False) == cp.CP_ERR_SHAPE


def test_null_pointers_and_missing_workspace_are_rejected_before_any_launch(lib):
    ok = _shape([32], [32], Hq=4, Hkv=2, splits=2)
    assert cp.cp_extend_attention(None, 1, 1, 1, 1, 1, 1, 1, None, ok, None, 0,
                                  check=False) == cp.CP_ERR_NULL
    assert cp.cp_extend_attention(1, 1, 1, 1, None, 1, 1, 1, None, ok, None, 0,
                                  check=False) == cp.CP_ERR_NULL
    assert cp.cp_extend_attention(256, 256, 256, 256, 256, 256, 256, 256, None, ok, None, 0,
                                  check=False) == cp.CP_ERR_WORKSPACE
    assert cp.cp_extend_attention(256, 256, 256, 256, 256, 256, 256, 256, None, ok, 128, 1 << 30,
                                  check=False) == cp.CP_ERR_WORKSPACE      # misaligned
    assert cp.cp_write_kv(None, 1, 1, 1, 1, 1, None, ok, check=False) == cp.CP_ERR_NULL
    with pytest.raises(cp.CpError):
        cp.cp_write_kv(None, 1, 1, 1, 1, 1, None, ok)


def test_misaligned_device_pointers_are_rejected_before_any_launch(lib):
    """q, k_new, v_new, kv_pages and out are moved in 16-byte pieces, the int32 arrays in 4-byte
    ones: every pointer is checked on the host, one at a time here."""
    ok = _shape([32], [32], Hq=4, Hkv=2, splits=1)
    base = [4096] * 8                      # q, k_new, v_new, kv_pages, table, prefix, extend, out
    for slot in (0, 1, 2, 3, 7):
        for off in (2, 8):
            args = list(base)
            args[slot] += off
            assert cp.cp_extend_attention(*args, None, ok, None, 0, check=False) == cp.CP_ERR_ALIGN
    for slot in (4, 5, 6):
        args = list(base)
        args[slot] += 2
        assert cp.cp_extend_attention(*args, None, ok, None, 0, check=False) == cp.CP_ERR_ALIGN
    wbase = [4096] * 6                     # k_new, v_new, kv_pages, table, prefix, extend
    for slot, off in ((0, 8), (1, 4), (2, 2), (3, 1), (4, 2), (5, 3)):
        args = list(wbase)
        args[slot] += off
        assert cp.cp_write_kv(*args, None, ok, check=False) == cp.CP_ERR_ALIGN
    st, info = cp.cp_check_tables(4098, 4096, 4096, None, ok, check=False)
    assert st == cp.CP_ERR_ALIGN and info == [-1, -1, -1]
    st, _ = cp.cp_check_tables(None, 4096, 4096, None, ok, check=False)
    assert st == cp.CP_ERR_NULL


def test_empty_batch_is_a_no_op(lib):
    sh = _shape([16, 0], [0, 0], Hq=4, Hkv=2)
    assert cp.cp_extend_attention(None, None, None, None, 1, 1, 1, None, None, sh, None, 0,
                                  check=False) == cp.CP_OK
    assert cp.cp_write_kv(None, None, None, 1, 1, 1, None, sh, check=False) == cp.CP_OK


def test_context_distance_argument_checks(lib):
    f = cp.cp_context_distance
    assert f(1, 1, -1, 16, 0.001, 1, None, check=False) == -2
    assert f(1, 1, 10, 0, 0.001, 1, None, check=False) == -2
    assert f(1, 1, 10, 33, 0.001, 1, None, check=False) == -2
    assert f(1, 1, 10, 6, 0.001, 1, None, check=False) == -2            # stride not a multiple of 4
    assert f(1, 1, 10, 16, -1.0, 1, None, check=False) == -2
    assert f(None, 1, 10, 16, 0.001, 1, None, check=False) == -1
    assert f(None, None, 0, 16, 0.001, None, None, check=False) == 0     # nothing to do
