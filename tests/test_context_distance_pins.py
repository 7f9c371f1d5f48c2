"""Pins of the context-distance oracle (paper, Section 4.1, Eq. 1) against the paper's own
worked examples (tests/golden/context_distance_examples.txt), hand evaluation of Eq. 1,
invariants, and a brute-force set formulation in Python."""
import os

import numpy as np
import pytest

import oracle
import workloads as W

ALPHA = 0.001
HERE = os.path.dirname(os.path.abspath(__file__))


def _dist(lists, alpha=ALPHA):
    k = max(len(l) for l in lists)
    C = np.full((len(lists), max(k, 1)), -1, np.int32)
    for i, l in enumerate(lists):
        C[i, :len(l)] = l
    return oracle.context_distance(C, np.array([len(l) for l in lists], np.int32), alpha)


def _golden():
    named, facts = {}, []
    for line in open(os.path.join(HERE, "golden", "context_distance_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a, b, fact = [x.strip() for x in line.split("|")]
        (na, ia), (nb, ib) = a.split(), b.split()
        named[na] = [int(x) for x in ia.split(",")]
        named[nb] = [int(x) for x in ib.split(",")]
        facts.append((na, nb, fact.split()))
    return named, facts


def test_paper_worked_examples():
    named, facts = _golden()
    # contexts that only appear on the right-hand side of a "less_than"
    named.setdefault("C3", [4, 1, 0])
    names = sorted(named)
    D = _dist([named[n] for n in names])
    D0 = _dist([named[n] for n in names], alpha=0.0)      # overlap-only metric
    ix = {n: i for i, n in enumerate(names)}
    for na, nb, (kind, arg) in facts:
        if kind == "overlap_only":
            assert D0[ix[na], ix[nb]] == pytest.approx(float(arg), abs=1e-15)
        else:
            oa, ob = arg.split("-")
            assert D[ix[na], ix[nb]] < D[ix[oa], ix[ob]]


def test_hand_evaluation_of_eq1():
    A, B, C, Dd = [3, 5, 1, 7], [2, 6, 3, 5], [3, 5, 8, 9], [2, 6, 4, 0]
    D = _dist([A, B, C, Dd])
    # A-B share {3,5} at positions (0,1) vs (2,3): 1 - 2/4 + alpha * (2 + 2) / 2
    assert D[0, 1] == pytest.approx(0.5 + 2 * ALPHA, abs=1e-15)
    assert D[1, 2] == pytest.approx(0.5 + 2 * ALPHA, abs=1e-15)
    assert D[1, 3] == pytest.approx(0.5, abs=1e-15)         # {2,6} at the same positions
    assert D[0, 3] == 1.0 and D[2, 3] == 1.0                # nothing shared
    assert D[0, 2] == pytest.approx(0.5, abs=1e-15)         # {3,5} at positions 0,1 in both
    # different lengths: max(|Ci|,|Cj|) in the denominator
    E = _dist([[1, 2, 3, 4, 5, 6], [9, 1]])
    assert E[0, 1] == pytest.approx(1 - 1 / 6 + ALPHA * 1.0, abs=1e-15)


def test_invariants():
    C, L = W.make_contexts(5, 60, (3, 12), pool_ids=40)
    D = oracle.context_distance(C, L, 0.01)
    np.testing.assert_array_equal(D, D.T)                    # symmetric
    np.testing.assert_array_equal(np.diag(D), 0.0)           # identical context: 0
    assert (D >= 0).all() and (D <= 1 + 0.01 * 12).all()
    # a permuted copy shares everything: only the positional term is left
    perm = C[0, :L[0]][::-1].copy()
    C2 = np.vstack([C[:1], np.pad(perm, (0, C.shape[1] - len(perm)), constant_values=-1)[None]])
    D2 = oracle.context_distance(C2, np.array([L[0], L[0]], np.int32), 0.01)
    n = int(L[0])
    gap = sum(abs(a - (n - 1 - a)) for a in range(n))
    assert D2[0, 1] == pytest.approx(0.01 * gap / n, abs=1e-15)
    # relabelling the block ids changes nothing
    relabel = np.random.default_rng(0).permutation(40).astype(np.int32)
    C3 = np.where(C >= 0, relabel[np.maximum(C, 0)], -1)
    np.testing.assert_array_equal(oracle.context_distance(C3, L, 0.01), D)


def test_brute_force_with_python_sets():
    C, L = W.make_contexts(6, 40, (1, 9), pool_ids=25)
    D = oracle.context_distance(C, L, ALPHA)
    for i in range(40):
        ci = C[i, :L[i]].tolist()
        for j in range(40):
            cj = C[j, :L[j]].tolist()
            S = set(ci) & set(cj)
            if not S:
                want = 1.0
            else:
                want = 1 - len(S) / max(len(ci), len(cj)) + \
                    ALPHA * sum(abs(ci.index(k) - cj.index(k)) for k in S) / len(S)
            assert D[i, j] == pytest.approx(want, abs=1e-14)


def test_generator_gives_distinct_ids_and_heavy_tail():
    C, L = W.make_contexts(7, 500, 15, pool_ids=2000, stride=16)
    assert C.shape == (500, 16) and (L == 15).all() and (C[:, 15] == -1).all()
    for i in range(500):
        row = C[i, :15]
        assert len(set(row.tolist())) == 15 and row.min() >= 0 and row.max() < 2000
    # the most popular 20 % of the ids cover most of the draws (paper: 50-80 %)
    counts = np.bincount(C[C >= 0], minlength=2000)
    assert np.sort(counts)[::-1][:400].sum() / counts.sum() > 0.5
    C2, _ = W.make_contexts(7, 500, 15, pool_ids=2000, stride=16)
    np.testing.assert_array_equal(C, C2)
