"""Oracle of DR-SpMM with degree-adaptive K (paper Section 3.2, Alg. 1 stage 2 and the text after it: neighbour
groups are classified by degree into low / medium / high, and D-ReLU applies K1 > K2 > K3 to them -- the more
neighbours a destination has, the fewer entries of each neighbour's embedding it receives), in fp64 numpy.

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and by nothing in the GPU package).

Reading (the paper gives neither the class boundaries nor the K values, and no formula):
  * the class of a neighbour group is decided by the in-degree of its DESTINATION row i in that relation:
        K(i) = k1 if deg(i) <= t1,   k2 if t1 < deg(i) <= t2,   k3 otherwise,        k1 >= k2 >= k3 >= 1;
  * destination i aggregates the top-K(i) entries of every neighbour's embedding row:
        H[i, :] = sum over edges (i <- j) of a_ij * f_{K(i)}(X_j);
  * f_K keeps the K largest signed values of a row, ties to the lower column, so the selections are nested and a
    row-sparse operand stored in RANK order (largest value first) holds every f_K, K <= k1, as a prefix;
  * the backward is the derivative of that forward with the selections held fixed, in the same rank order:
        G[j, t] = sum over edges (i <- j) with t < K(i) of a_ij * dH[i, col(j, t)],   col(j, t) = column of the
        t-th largest entry of X_j.
With k1 = k2 = k3 this is the uniform-K DR-SpMM (rank order instead of ascending columns).
"""
from __future__ import annotations

from typing import NamedTuple

import numpy as np


class DegreeClasses(NamedTuple):
    t1: int
    t2: int
    k1: int
    k2: int
    k3: int

    def k_of_degree(self, deg):
        deg = np.asarray(deg)
        return np.where(deg <= self.t1, self.k1, np.where(deg <= self.t2, self.k2, self.k3)).astype(np.int64)


def topk_ranked(X, k: int):
    """Row-wise D-ReLU in rank order: columns ordered by (value descending, column ascending), first k kept.
    Returns (vals[n,k] fp64 copies of the inputs, idx[n,k] int32).  -0.0 and +0.0 compare equal."""
    X = np.asarray(X, dtype=np.float64)
    if not np.all(np.isfinite(X)):
        raise ValueError("non-finite input")
    n, D = X.shape
    if not 1 <= k <= D:
        raise ValueError("k out of range")
    key = X + 0.0                                     # -0.0 -> +0.0
    cols = np.broadcast_to(np.arange(D), (n, D))
    order = np.lexsort((cols, -key), axis=1)[:, :k]   # last key is the primary one
    return np.take_along_axis(X, order, axis=1), order.astype(np.int32)


def _edges(rowptr, colidx):
    rowptr = np.asarray(rowptr, dtype=np.int64)
    deg = np.diff(rowptr)
    rows = np.repeat(np.arange(deg.shape[0]), deg)
    return rows, np.asarray(colidx, dtype=np.int64), deg


def spmm_fwd_adaptive(rowptr, colidx, avals, xr_vals, xr_idx, D: int, cls: DegreeClasses):
    """H[M,D] and, per element, the sum of |terms| (for the error bound).  (xr_vals, xr_idx): rank-ordered CBSR of
    the source rows at width k1."""
    rows, cols, deg = _edges(rowptr, colidx)
    a = np.asarray(avals, dtype=np.float64)
    xr_vals, xr_idx = np.asarray(xr_vals, dtype=np.float64), np.asarray(xr_idx, dtype=np.int64)
    assert xr_vals.shape[1] == cls.k1
    M = deg.shape[0]
    H, L1 = np.zeros((M, D)), np.zeros((M, D))
    k_edge = cls.k_of_degree(deg)[rows]                       # K of the destination of every edge
    for t in range(cls.k1):                                   # t-th largest entry of every source row
        use = k_edge > t
        term = a[use] * xr_vals[cols[use], t]
        np.add.at(H, (rows[use], xr_idx[cols[use], t]), term)
        np.add.at(L1, (rows[use], xr_idx[cols[use], t]), np.abs(term))
    return H, L1


def spmm_bwd_adaptive(rowptr, colidx, avals, dH, xr_idx, n_src: int, cls: DegreeClasses):
    """G[N,k1] in rank order and the per-element sum of |terms|, from the FORWARD CSR (rows = destinations)."""
    rows, cols, deg = _edges(rowptr, colidx)
    a = np.asarray(avals, dtype=np.float64)
    dH = np.asarray(dH, dtype=np.float64)
    xr_idx = np.asarray(xr_idx, dtype=np.int64)
    G, L1 = np.zeros((n_src, cls.k1)), np.zeros((n_src, cls.k1))
    k_edge = cls.k_of_degree(deg)[rows]
    for t in range(cls.k1):
        use = k_edge > t
        term = a[use] * dH[rows[use], xr_idx[cols[use], t]]
        np.add.at(G[:, t], cols[use], term)
        np.add.at(L1[:, t], cols[use], np.abs(term))
    return G, L1
