"""The C++ context index (through the C ABI) against the Python oracle: same trees, aligned
contexts, search paths and schedules, node for node.  Integer and structural work: the bar is
exact equality (clustering distances are combined in double precision on both sides).  Host
code only: these tests need no GPU."""
import os

import numpy as np
import pytest

import oracle
from oracle import context_index as CI
import paper_2511_03475_amd as cp
import workloads as W

ALPHA = 0.001
HERE = os.path.dirname(os.path.abspath(__file__))


def _pack(contexts, stride=None):
    stride = stride or max([len(c) for c in contexts] + [1])
    C = np.full((max(len(contexts), 1), stride), -1, np.int32)
    L = np.zeros(max(len(contexts), 1), np.int32)
    for i, c in enumerate(contexts):
        C[i, :len(c)] = c
        L[i] = len(c)
    return C[:len(contexts)].reshape(len(contexts), stride), L[:len(contexts)]


def _same_tree(idx: cp.ContextIndex, ref: CI.ContextIndex):
    """Walks both trees from the root in lock step."""
    stack = [(0, ref.root)]
    seen = 0
    while stack:
        h, v = stack.pop()
        got = idx.node(h)
        seen += 1
        assert got["docs"] == v.docs and got["leaf"] == v.leaf and got["freq"] == v.freq, (h, got, v.docs)
        assert got["created_at"] == v.created_at
        kids = idx.children(h)
        assert len(kids) == len(v.children) == got["num_children"]
        if v.parent is None:
            assert got["parent"] == -1
        for k, c in zip(kids, v.children):
            assert idx.node(k)["parent"] == h
            stack.append((k, c))
    return seen


def _same_contexts(idx, ref, n):
    assert idx.num_contexts() == len(ref.leaf_of) == n
    for i in range(n):
        assert idx.aligned(i) == ref.aligned(i), i
        assert idx.path(i) == ref.path(i), i


def test_paper_worked_example_through_the_c_abi():
    C, L = _pack([[2, 1, 3], [2, 6, 1], [4, 1, 0]])
    idx = cp.ContextIndex(C, L, ALPHA)
    assert [idx.aligned(i) for i in range(3)] == [[1, 2, 3], [1, 2, 6], [1, 4, 0]]
    assert [idx.path(i) for i in range(3)] == [[0, 0, 0], [0, 0, 1], [0, 1]]
    c5 = idx.children(0)
    assert len(c5) == 1 and idx.node(c5[0])["docs"] == [1]
    c4 = idx.children(c5[0])[0]
    assert idx.node(c4)["docs"] == [1, 2] and not idx.node(c4)["leaf"]
    path, node = idx.search([2, 1, 4])
    assert path == [0, 0] and node == c4
    a6, p6 = idx.insert([2, 1, 4])
    a7, p7 = idx.insert([5, 7, 8])
    a8, p8 = idx.insert([1, 2, 9])
    assert (a6, p6) == ([1, 2, 4], [0, 0, 2])
    assert (a7, p7) == ([5, 7, 8], [1])
    assert (a8, p8) == ([1, 2, 9], [0, 0, 3])
    order = cp.cp_index_schedule([p6, idx.path(2), p7, p8])      # C6, C3, C7, C8
    assert order == [0, 3, 1, 2]                                 # C6, C8, C3, C7
    idx.close()


@pytest.mark.parametrize("seed,n,k,pool", [(1, 12, 4, 10), (2, 60, 6, 30), (3, 150, 10, 200), (4, 40, 5, 6),
                                           (5, 300, 15, 2000)])
def test_build_matches_oracle_node_for_node(seed, n, k, pool):
    C, L = W.make_contexts(seed, n, k, pool_ids=pool, stride=16)
    contexts = [list(map(int, C[i, :L[i]])) for i in range(n)]
    ref = CI.ContextIndex.build(contexts, ALPHA)
    idx = cp.ContextIndex(C, L, ALPHA)
    reachable = _same_tree(idx, ref)
    assert reachable == len(ref.nodes_bfs())
    _same_contexts(idx, ref, n)
    paths = [ref.path(i) for i in range(n)]
    assert cp.cp_index_schedule(paths) == CI.schedule(paths)
    idx.close()


def test_build_from_a_given_float32_distance_matrix():
    """The distances may come from the GPU kernel as float32: both sides then cluster the same
    numbers."""
    n = 120
    C, L = W.make_contexts(8, n, 8, pool_ids=60, stride=8)
    first_of, m = cp.cp_index_distinct(C, L)
    rows = [int(np.flatnonzero(first_of == u)[0]) for u in range(m)]
    D = oracle.context_distance(C[rows], L[rows], ALPHA).astype(np.float32)
    contexts = [list(map(int, C[i, :L[i]])) for i in range(n)]
    ref = CI.ContextIndex.build(contexts, ALPHA, D=D.astype(np.float64).tolist())
    idx = cp.ContextIndex(C, L, ALPHA, dist=D)
    _same_tree(idx, ref)
    _same_contexts(idx, ref, n)
    with pytest.raises(cp.CpError):
        cp.ContextIndex(C, L, ALPHA, dist=D[:-1, :-1])           # wrong size
    idx.close()


def test_duplicates_and_distinct():
    contexts = [[3, 1, 2], [7, 8], [3, 1, 2], [3, 1, 2], [8, 7], []]
    C, L = _pack(contexts, 4)
    first_of, m = cp.cp_index_distinct(C, L)
    assert list(first_of) == [0, 1, 0, 0, 2, 3] and m == 4
    ref = CI.ContextIndex.build(contexts, ALPHA)
    idx = cp.ContextIndex(C, L, ALPHA)
    _same_tree(idx, ref)
    _same_contexts(idx, ref, len(contexts))
    assert idx.leaf(0) == idx.leaf(2) == idx.leaf(3) != idx.leaf(1)
    idx.close()


@pytest.mark.parametrize("seed,pool", [(11, 25), (12, 8), (13, 400)])
def test_insert_sequence_matches_oracle_step_by_step(seed, pool):
    C, L = W.make_contexts(seed, 90, 6, pool_ids=pool, stride=8)
    contexts = [list(map(int, C[i, :L[i]])) for i in range(90)]
    ref = CI.ContextIndex.build(contexts[:30], ALPHA)
    idx = cp.ContextIndex(C[:30], L[:30], ALPHA)
    for c in contexts[30:]:
        want_path, want_node = ref.search(c)
        got_path, got_node = idx.search(c)
        assert got_path == want_path and idx.node(got_node)["docs"] == want_node.docs
        assert idx.insert(c) == ref.insert(c)
    _same_tree(idx, ref)
    _same_contexts(idx, ref, 90)
    idx.close()


def test_empty_batch_then_inserts():
    C = np.zeros((0, 4), np.int32)
    idx = cp.ContextIndex(C, np.zeros(0, np.int32), ALPHA)
    ref = CI.ContextIndex.build([], ALPHA)
    assert idx.num_contexts() == 0 and idx.num_nodes() == 1
    for c in ([4, 5], [4, 6], [9], [4, 5]):
        assert idx.insert(c) == ref.insert(c)
    _same_tree(idx, ref)
    idx.close()


def test_error_paths():
    lib = cp.load_library()
    C, L = _pack([[1, 2], [2, 2]])                               # repeated id in a row
    with pytest.raises(cp.CpError):
        cp.ContextIndex(C, L, ALPHA)
    C, L = _pack([[1, 2], [3, -4]])                              # negative id
    with pytest.raises(cp.CpError):
        cp.ContextIndex(C, L, ALPHA)
    C, L = _pack([[1, 2], [3, 4]])
    with pytest.raises(cp.CpError):
        cp.ContextIndex(C, np.array([2, 3], np.int32), ALPHA)    # length beyond the stride
    with pytest.raises(cp.CpError):
        cp.ContextIndex(C, L, -1.0)
    idx = cp.ContextIndex(C, L, ALPHA)
    with pytest.raises(cp.CpError):
        idx.aligned(2)
    with pytest.raises(cp.CpError):
        idx.node(99)
    with pytest.raises(cp.CpError):
        idx.insert([5, 5])
    assert lib.cp_index_num_contexts(None) == -1
    idx.close()


def test_schedule_matches_oracle_on_random_paths():
    rng = np.random.default_rng(0)
    for _ in range(20):
        n = int(rng.integers(0, 40))
        paths = [list(map(int, rng.integers(0, 4, size=int(rng.integers(0, 5))))) for _ in range(n)]
        assert cp.cp_index_schedule(paths) == CI.schedule(paths)
