"""Helpers shared by the GPU parity tests (host <-> device plumbing and the tolerance checks)."""
import sys

import numpy as np
import torch

# fp32 result vs fp64 oracle: the contract is max|err| <= 1e-4 * (row L1 norm of the contributing
# terms).  The per-element check is the stricter one the arithmetic supports: fp32 accumulation of n
# terms is off by at most about n * 2^-24 * sum|terms|, far below 1e-5 * sum|terms| for n <= a few hundred,
# and exactly zero where no term contributes.
ROW_TOL = 1e-4
ELEM_TOL = 1e-5


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def host_idx(t):
    """uint16 CBSR indices live in an int16 torch tensor; view them back as unsigned."""
    return t.cpu().numpy().view(np.uint16).astype(np.int32)


def assert_row_bound(got, want, l1row, what, tol=ROW_TOL):
    err = np.abs(got.astype(np.float64) - want)
    worst = err.max(axis=1) if err.ndim == 2 else err
    bad = worst > tol * l1row + 1e-30
    assert not bad.any(), (what, int(bad.sum()), float((worst / np.maximum(l1row, 1e-300)).max()))
    return float((worst / np.maximum(l1row, 1e-300)).max())


def assert_elem_bound(got, want, l1elem, what, tol=ELEM_TOL):
    err = np.abs(got.astype(np.float64) - want)
    bad = err > tol * l1elem
    assert not bad.any(), (what, int(bad.sum()), float(err.max()))
    zero = l1elem == 0
    assert np.all(got[zero] == 0), (what, "non-zero output where no term contributes")


def cells_with_agreeing_masks(near_rowptr, near_colidx, mask_a, mask_b):
    """Cells whose input gradient does not depend on a max-merge decision on which the two masks differ: the cell's own
    row and the rows of every `near` destination it feeds agree (near: rows = destinations, columns = sources)."""
    row_bad = (mask_a != mask_b).any(axis=1)
    dst = np.repeat(np.arange(len(row_bad)), np.diff(near_rowptr.astype(np.int64)))
    feeds_bad = np.zeros(len(row_bad), np.int64)
    np.add.at(feeds_bad, near_colidx.astype(np.int64), row_bad[dst].astype(np.int64))
    return ~row_bad & (feeds_bad == 0)


def random_csr(rng, M, N, max_deg, dup=False, empty_frac=0.2, evil_rows=(), evil_deg=0):
    deg = rng.integers(0, max_deg + 1, size=M)
    deg[rng.random(M) < empty_frac] = 0
    for r in evil_rows:
        deg[r] = evil_deg
    rowptr = np.zeros(M + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum(deg)
    if dup:
        colidx = rng.integers(0, N, size=int(rowptr[-1])).astype(np.int32)
    else:
        parts = [rng.permutation(N)[:d] if d <= N else rng.integers(0, N, size=d) for d in deg]
        colidx = (np.concatenate(parts) if parts else np.zeros(0)).astype(np.int32)
    vals = rng.uniform(0.05, 1.0, size=colidx.shape[0]).astype(np.float32)
    return rowptr, colidx, vals


class HostPattern:
    def __init__(self, n_rows, n_cols, rowptr, colidx):
        self.n_rows, self.n_cols, self.rowptr, self.colidx = n_rows, n_cols, rowptr, colidx
