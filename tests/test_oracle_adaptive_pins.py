"""Pins of the degree-adaptive-K oracle (oracle/adaptive.py) against things other than itself: the definition
written out densely row by row with a stable sort, the independently pinned uniform-K oracle where the three K
coincide, central differences of a scalar functional, and the prefix property of the rank order."""
import numpy as np
import pytest

import oracle
from oracle import adaptive as oad
from gpu_util import random_csr


def _case(seed, M=60, N=45, D=16, max_deg=9, evil=True):
    rng = np.random.default_rng(seed)
    rowptr, colidx, avals = random_csr(rng, M, N, max_deg, dup=True, evil_rows=(3, 17) if evil else (), evil_deg=40)
    X = rng.standard_normal((N, D))
    X[5, :4] = 0.5                                    # ties inside a row
    X[7, 2] = -0.0
    X[7, 9] = 0.0
    return rowptr, colidx, avals, X, rng


def _dense_topk(x, K):
    """f_K(x) as a dense row: stable sort of -x puts equal values in column order."""
    keep = np.argsort(-(x + 0.0), kind="stable")[:K]
    out = np.zeros_like(x)
    out[keep] = x[keep]
    return out


@pytest.mark.parametrize("cls", [oad.DegreeClasses(3, 7, 8, 5, 2), oad.DegreeClasses(0, 20, 16, 3, 1),
                                 oad.DegreeClasses(4, 4, 6, 6, 1)])
def test_forward_is_the_row_by_row_definition(cls):
    rowptr, colidx, avals, X, rng = _case(1)
    D = X.shape[1]
    xv, xi = oad.topk_ranked(X, cls.k1)
    H, L1 = oad.spmm_fwd_adaptive(rowptr, colidx, avals, xv, xi, D, cls)
    want = np.zeros_like(H)
    for i in range(len(rowptr) - 1):
        deg = rowptr[i + 1] - rowptr[i]
        K = cls.k1 if deg <= cls.t1 else (cls.k2 if deg <= cls.t2 else cls.k3)
        for e in range(rowptr[i], rowptr[i + 1]):
            want[i] += float(avals[e]) * _dense_topk(X[colidx[e]], K)
    np.testing.assert_allclose(H, want, rtol=0, atol=1e-12)
    assert np.all(L1 >= np.abs(H) - 1e-12)
    # all three classes occur in this graph
    deg = np.diff(rowptr)
    assert len({int(k) for k in cls.k_of_degree(deg)}) == len({cls.k1, cls.k2, cls.k3})


def test_equal_k_is_the_uniform_dr_spmm():
    rowptr, colidx, avals, X, rng = _case(2)
    M, (N, D), k = len(rowptr) - 1, X.shape, 5
    cls = oad.DegreeClasses(2, 6, k, k, k)
    xv, xi = oad.topk_ranked(X, k)
    av, ai = oracle.topk(X, k)                                    # ascending-column CBSR of the same selection
    assert np.array_equal(np.sort(xi, axis=1), ai)
    H, _ = oad.spmm_fwd_adaptive(rowptr, colidx, avals, xv, xi, D, cls)
    H0, _ = oracle.spmm_fwd(rowptr, colidx, avals, av, ai, D)
    np.testing.assert_allclose(H, H0, rtol=0, atol=1e-12)
    dH = rng.standard_normal((M, D))
    G, _ = oad.spmm_bwd_adaptive(rowptr, colidx, avals, dH, xi, N, cls)
    t = oracle.csr_transpose(M, N, rowptr, colidx, avals)
    G0, _ = oracle.spmm_bwd(*t, dH, ai)
    # same gradients, listed in rank order instead of column order
    pos = np.argsort(xi, axis=1, kind="stable")
    np.testing.assert_allclose(np.take_along_axis(G, pos, axis=1), G0, rtol=0, atol=1e-12)


def test_backward_is_the_derivative_of_the_forward():
    rowptr, colidx, avals, X, rng = _case(3)
    M, (N, D) = len(rowptr) - 1, X.shape
    cls = oad.DegreeClasses(3, 7, 8, 4, 2)
    R = rng.standard_normal((M, D))

    def functional(Xp):
        xv, xi = oad.topk_ranked(Xp, cls.k1)
        return float(np.sum(oad.spmm_fwd_adaptive(rowptr, colidx, avals, xv, xi, D, cls)[0] * R))

    h = 1e-6
    X = X.copy()
    X[5, :4] += np.array([4e-3, 3e-3, 2e-3, 1e-3])    # break the planted ties: the selection must not move under +-h
    X[7, 2], X[7, 9] = -1e-3, 2e-3
    xv, xi = oad.topk_ranked(X, cls.k1)
    G, _ = oad.spmm_bwd_adaptive(rowptr, colidx, avals, R, xi, N, cls)
    dense = np.zeros((N, D))
    np.put_along_axis(dense, xi.astype(np.int64), G, axis=1)
    for trial in range(4):
        d = rng.standard_normal(X.shape)
        fd = (functional(X + h * d) - functional(X - h * d)) / (2 * h)
        an = float(np.sum(dense * d))
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (trial, fd, an)
    # entry by entry on two source rows: a column kept only at the larger widths gets gradient from the low-degree
    # destinations alone
    for j in (0, 11):
        for c in range(D):
            E = np.zeros_like(X)
            E[j, c] = h
            fd = (functional(X + E) - functional(X - E)) / (2 * h)
            assert abs(fd - dense[j, c]) <= 1e-6 * max(1.0, abs(fd)), (j, c)


def test_rank_order_prefixes_are_the_smaller_selections():
    rowptr, colidx, avals, X, rng = _case(4)
    v8, i8 = oad.topk_ranked(X, 8)
    for k in (1, 3, 8):
        vk, ik = oad.topk_ranked(X, k)
        assert np.array_equal(ik, i8[:, :k]) and np.array_equal(vk, v8[:, :k])
        assert np.array_equal(np.sort(ik, axis=1), oracle.topk(X, k)[1])
    assert np.all(np.diff(v8, axis=1) <= 0)                       # descending values
    tie = np.where(v8[5] == 0.5)[0]        # planted tie of columns 0..3: those that fit are the lowest, in column order
    assert len(tie) >= 2 and list(i8[5, tie]) == list(range(len(tie)))
    # signed zeros compare equal: the lower column comes first
    z = np.where(np.isin(i8[7], (2, 9)))[0]
    if len(z) == 2:
        assert i8[7, z[0]] == 2
