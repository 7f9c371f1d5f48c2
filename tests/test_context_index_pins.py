"""Pins of the context-index oracle (paper, Sections 4-5 and the appendix algorithms) against
the paper's own worked examples (tests/golden/context_index_examples.txt), a library routine
for the clustering step, and invariants that any correct index must keep."""
import os

import numpy as np
import pytest

import oracle
from oracle import context_index as CI
import workloads as W

ALPHA = 0.001
HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    facts = []
    for line in open(os.path.join(HERE, "golden", "context_index_examples.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            facts.append([x.strip() for x in line.split("|")])
    return facts


def _ids(s):
    return [int(x) for x in s.split(",")] if s else []


def test_paper_worked_example_end_to_end():
    facts = _golden()
    ctx = {f[1]: _ids(f[2]) for f in facts if f[0] == "context"}
    idx = CI.ContextIndex.build([ctx["C1"], ctx["C2"], ctx["C3"]], ALPHA)
    leaf = {"C1": idx.leaf_of[0], "C2": idx.leaf_of[1], "C3": idx.leaf_of[2]}
    # virtual nodes: found by their children
    for f in facts:
        if f[0] != "virtual":
            continue
        kids = f[3].split()[1].split(",")
        node = leaf[kids[0]].parent if kids[0] in leaf else None
        if node is None:        # first child is itself virtual (C4 under C5)
            node = virtual[kids[0]].parent
        virtual = locals().get("virtual", {})
        virtual[f[1]] = node
        assert node.docs == _ids(f[2]), f
        got = [("leaf", id(c)) if c.leaf else ("virt", id(c)) for c in node.children]
        want = [("leaf", id(leaf[k])) if k in leaf else ("virt", id(virtual[k])) for k in kids]
        assert got == want, f
    assert virtual["C5"].parent is idx.root and idx.root.docs == []
    aligned = {"C1": idx.aligned(0), "C2": idx.aligned(1), "C3": idx.aligned(2)}
    paths = {"C3": idx.path(2)}
    for f in facts:
        if f[0] == "search":
            assert idx.search(ctx[f[1]])[0] == _ids(f[2]), f
            assert idx.search(ctx[f[1]])[1] is virtual["C4"]
    for name in ("C6", "C7", "C8"):
        aligned[name], paths[name] = idx.insert(ctx[name])
    for f in facts:
        if f[0] == "aligned":
            assert aligned[f[1]] == _ids(f[2]), f
        if f[0] == "path":
            assert paths[f[1]] == _ids(f[2]), f
        if f[0] == "schedule":
            names = f[1].split(",")
            order = CI.schedule([paths[n] for n in names])
            assert [names[i] for i in order] == f[2].split(","), f


def test_distance_agrees_with_the_matrix_oracle():
    """Two independent writings of Eq. 1 (C with position tables, Python with dictionaries)."""
    C, L = W.make_contexts(5, 60, 9, pool_ids=40, stride=12)
    lists = [list(C[i, :L[i]]) for i in range(len(L))]
    D = oracle.context_distance(C, L, ALPHA)
    for i in range(0, 60, 7):
        for j in range(60):
            want = 0.0 if i == j else CI.distance(lists[i], lists[j], ALPHA)
            assert abs(D[i, j] - want) < 1e-12


def test_linkage_matches_library_average_linkage_when_there_are_no_ties():
    from scipy.cluster.hierarchy import linkage as sp_linkage
    from scipy.spatial.distance import squareform
    rng = np.random.default_rng(3)
    for n in (2, 3, 9, 40):
        X = rng.random((n, n))
        D = (X + X.T) / 2
        np.fill_diagonal(D, 0.0)
        Z = sp_linkage(squareform(D, checks=False), method="average")
        mine = CI.linkage(D.tolist())
        assert len(mine) == n - 1
        for (a, b, d, size), z in zip(mine, Z):
            assert {a, b} == {int(z[0]), int(z[1])}
            assert abs(d - z[2]) < 1e-12 and size == int(z[3])


def test_linkage_tie_rule_and_hand_example():
    # four points on a line at 0, 1, 2, 4: (0,1) and (1,2) tie at 1 -> lowest pair first
    pts = [0.0, 1.0, 2.0, 4.0]
    D = [[abs(a - b) for b in pts] for a in pts]
    assert CI.linkage(D) == [(0, 1, 1.0, 2), (2, 4, 1.5, 3), (3, 5, 3.0, 4)]


def _check_tree(idx, contexts):
    nodes = idx.nodes_bfs()
    assert nodes[0] is idx.root and idx.root.docs == [] and idx.root.parent is None
    for v in nodes[1:]:
        assert v.parent is not None and v in v.parent.children
        # the parent's context is a prefix of the node's
        assert v.docs[:len(v.parent.docs)] == v.parent.docs
        assert len(set(v.docs)) == len(v.docs)
        if v.leaf:
            assert not v.children and v.freq >= 1
        else:
            assert len(v.children) >= 2 and v.docs, "virtual nodes are shared, non-empty prefixes"
            # a virtual node holds exactly what all leaves below it share ... at build time
    for i, c in enumerate(contexts):
        a = idx.aligned(i)
        assert sorted(a) == sorted(c), "alignment only reorders"
        leaf = idx.leaf_of[i]
        # walking the stored path from the root reaches the leaf
        v = idx.root
        for step in idx.path(i):
            v = v.children[step]
        assert v is leaf
        # blocks that were not inherited keep their original relative order
        inherited = set(leaf.parent.docs)
        assert [b for b in a if b not in inherited] == [b for b in c if b not in inherited]


@pytest.mark.parametrize("seed,n,k,pool", [(1, 12, 4, 10), (2, 40, 6, 30), (3, 80, 10, 200), (4, 30, 5, 6)])
def test_build_invariants_on_zipf_contexts(seed, n, k, pool):
    C, L = W.make_contexts(seed, n, k, pool_ids=pool, stride=12)
    contexts = [list(map(int, C[i, :L[i]])) for i in range(n)]
    idx = CI.ContextIndex.build(contexts, ALPHA)
    _check_tree(idx, contexts)
    # build-time virtual nodes hold exactly the blocks shared by every leaf below them
    for v in idx.nodes_bfs()[1:]:
        if not v.leaf:
            below = [set(x.docs) for x in idx.nodes_bfs() if x.leaf and _is_below(x, v)]
            assert set(v.docs) == set.intersection(*below)
    assert sum(x.freq for x in idx.nodes_bfs() if x.leaf) == n


def _is_below(x, v):
    while x is not None:
        if x is v:
            return True
        x = x.parent
    return False


def test_duplicates_share_a_leaf():
    contexts = [[3, 1, 2], [7, 8], [3, 1, 2], [3, 1, 2], [8, 7]]
    idx = CI.ContextIndex.build(contexts, ALPHA)
    assert idx.leaf_of[0] is idx.leaf_of[2] is idx.leaf_of[3] and idx.leaf_of[0].freq == 3
    assert idx.leaf_of[1] is not idx.leaf_of[4]          # same set, different order: not identical
    _check_tree(idx, contexts)
    a, p = idx.insert([3, 1, 2])
    assert idx.leaf_of[-1] is idx.leaf_of[0] and idx.leaf_of[0].freq == 4 and p == idx.path(0)


def test_disjoint_contexts_hang_under_the_root():
    contexts = [[1, 2], [3, 4], [5, 6]]
    idx = CI.ContextIndex.build(contexts, ALPHA)
    assert [c.docs for c in idx.root.children] and all(c.leaf for c in idx.root.children)
    assert sorted(idx.path(i)[0] for i in range(3)) == [0, 1, 2]
    assert all(idx.aligned(i) == contexts[i] for i in range(3))


def test_insert_matching_a_leaf_creates_a_virtual_node():
    idx = CI.ContextIndex.build([[1, 2, 3], [9, 8]], ALPHA)
    a, p = idx.insert([3, 1, 7])        # shares {1,3} with the only overlapping leaf
    leaf = idx.leaf_of[0]
    assert leaf.parent.docs == [1, 3] and not leaf.parent.leaf
    assert a == [1, 3, 7] and p == leaf.parent.path() + [1] and idx.path(0) == leaf.parent.path() + [0]
    assert leaf.docs == [1, 2, 3], "a cached leaf keeps its order"


def test_insert_sequence_keeps_invariants_and_paths():
    C, L = W.make_contexts(11, 50, 6, pool_ids=25, stride=8)
    contexts = [list(map(int, C[i, :L[i]])) for i in range(50)]
    idx = CI.ContextIndex.build(contexts[:20], ALPHA)
    for c in contexts[20:]:
        a, p = idx.insert(c)
        assert sorted(a) == sorted(c)
        v = idx.root
        for step in p:
            v = v.children[step]
        assert v is idx.leaf_of[-1]
        # the new leaf starts with its parent's context, and everything above it is part of c
        assert v.docs[:len(v.parent.docs)] == v.parent.docs
        anc = v.parent
        while anc is not None:
            assert set(anc.docs) <= set(c)
            anc = anc.parent
    for i in range(50):
        v = idx.root
        for step in idx.path(i):
            v = v.children[step]
        assert v is idx.leaf_of[i]


def test_schedule_rule_by_hand():
    paths = [[2, 0], [0, 1, 3], [2], [0, 4], [1], [2, 5, 6, 7], [0, 1, 2, 2]]
    # groups by first element: 2 -> [0,2,5], 0 -> [1,3,6], 1 -> [4]; equal sizes keep first-seen order
    assert CI.schedule(paths) == [5, 0, 2, 6, 1, 3, 4]
    assert CI.schedule([]) == []


def test_alignment_raises_exact_prefix_hits():
    """The point of the method (Section 3.1): aligned and scheduled contexts share longer exact
    prefixes than the contexts as retrieved."""
    C, L = W.make_contexts(7, 200, 10, pool_ids=300, stride=12)
    contexts = [list(map(int, C[i, :L[i]])) for i in range(200)]
    idx = CI.ContextIndex.build(contexts, ALPHA)
    aligned = [idx.aligned(i) for i in range(200)]
    order = CI.schedule([idx.path(i) for i in range(200)])
    base = sum(CI.prefix_hits(contexts, list(range(200))))
    ours = sum(CI.prefix_hits(aligned, order))
    assert sorted(order) == list(range(200))
    assert ours > 2 * base, (ours, base)


def test_prefix_hits_by_hand():
    assert CI.prefix_hits([[1, 2, 3], [1, 2, 4], [5], [1, 9]], [0, 1, 2, 3]) == [0, 2, 0, 1]
    assert CI.prefix_hits([[1, 2, 3], [1, 2, 4], [5], [1, 9]], [3, 1, 0, 2]) == [2, 1, 0, 0]
