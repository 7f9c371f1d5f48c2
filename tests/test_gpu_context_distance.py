"""GPU parity of cp_context_distance against the fp64 oracle (paper, Section 4.1, Eq. 1).

The shared count and the position gaps are integers and must agree exactly; the combination
1 - s/m + alpha * g/s is done in fp32 on the GPU, so values are compared to 4 fp32 ulps of 1
(4.8e-7); the diagonal must be exactly 0 and disjoint contexts exactly 1."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_03475_amd as cp
import workloads as W

pytestmark = pytest.mark.gpu
TOL = 4 * 2.0 ** -23


def _gpu(C, L, alpha):
    n, stride = C.shape
    dc = torch.from_numpy(np.ascontiguousarray(C)).to("cuda:0")
    dl = torch.from_numpy(np.ascontiguousarray(L)).to("cuda:0")
    out = torch.full((max(n, 1), max(n, 1)), -7.0, dtype=torch.float32, device="cuda:0")
    cp.cp_context_distance(dc, dl, n, stride, alpha, out, torch.cuda.current_stream())
    torch.cuda.synchronize()
    return out.cpu().numpy()[:n, :n].astype(np.float64)


def _check(C, L, alpha):
    got, want = _gpu(C, L, alpha), oracle.context_distance(C, L, np.float32(alpha))
    assert np.abs(got - want).max() <= TOL
    np.testing.assert_array_equal(np.diag(got), 0.0)
    np.testing.assert_array_equal(got, got.T)
    return got


def test_paper_example_on_gpu():
    C = np.full((4, 4), -1, np.int32)
    C[:] = [[3, 5, 1, 7], [2, 6, 3, 5], [3, 5, 8, 9], [2, 6, 4, 0]]
    D = _check(C, np.full(4, 4, np.int32), 0.001)
    assert D[1, 3] < D[0, 1] and D[1, 3] < D[1, 2] and D[1, 3] == 0.5


@pytest.mark.parametrize("n,k,stride", [(1, 5, 8), (255, 15, 16), (256, 3, 4), (1000, (1, 16), 16),
                                        (777, (0, 20), 20), (513, 32, 32), (300, (5, 15), 32)])
def test_random_contexts(n, k, stride):
    C, L = W.make_contexts(100 + n, n, k, pool_ids=200, stride=stride)
    _check(C, L, 0.01)


def test_all_equal_and_all_disjoint():
    C = np.tile(np.arange(15, dtype=np.int32), (300, 1))
    C = np.pad(C, ((0, 0), (0, 1)), constant_values=-1)
    np.testing.assert_array_equal(_check(C, np.full(300, 15, np.int32), 0.001), 0.0)
    C = np.arange(300 * 16, dtype=np.int32).reshape(300, 16)
    D = _check(C, np.full(300, 16, np.int32), 0.001)
    assert (D[~np.eye(300, dtype=bool)] == 1.0).all()


def test_index_scale_8k_contexts_sampled():
    """8192 contexts x top-15: the matrix is compared on a seeded sample of rows."""
    C, L = W.make_contexts(20251110, 8192, 15, pool_ids=2000, stride=16)
    got = _gpu(C, L, 0.001)
    rows = np.random.default_rng(1).choice(8192, size=64, replace=False)
    sub = np.vstack([C[rows], C])                    # oracle on (sample + all), take the block
    want = oracle.context_distance(sub, np.concatenate([L[rows], L]), np.float32(0.001))[:64, 64:]
    assert np.abs(got[rows] - want).max() <= TOL
