"""Pins for the CPU oracle: every oracle function is checked against something that is
not itself -- brute force in pure Python, dense numpy / scipy products, closed-form special
cases, the adjoint identity, torch.autograd on a dense re-formulation and central finite
differences.  No GPU needed."""
import itertools
import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from circuit_synth import make_graph, make_tensors
from circuit_synth.generate import transpose_pattern

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------------------
# helpers (test-local; plain numpy)
# ---------------------------------------------------------------------------

def random_csr(rng, M, N, max_deg, dup=False, empty_frac=0.2):
    """Random CSR with some empty rows; columns unsorted; optional duplicate entries."""
    deg = rng.integers(0, max_deg + 1, size=M)
    deg[rng.random(M) < empty_frac] = 0
    rowptr = np.zeros(M + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum(deg)
    cols = []
    for d in deg:
        if dup:
            cols.append(rng.integers(0, N, size=d))
        else:
            cols.append(rng.permutation(N)[:d] if d <= N else rng.integers(0, N, size=d))
    colidx = np.concatenate(cols).astype(np.int32) if cols else np.zeros(0, np.int32)
    vals = rng.uniform(0.1, 1.0, size=colidx.shape[0]).astype(np.float32)
    return rowptr, colidx, vals


def dense_of(rowptr, colidx, vals, M, N):
    A = np.zeros((M, N), dtype=np.float64)
    for i in range(M):
        for e in range(rowptr[i], rowptr[i + 1]):
            A[i, colidx[e]] += float(vals[e])
    return A


def brute_topk_row(row, k):
    order = sorted(range(len(row)), key=lambda c: (-float(row[c]), c))
    keep = sorted(order[:k])
    return keep


# ---------------------------------------------------------------------------
# O1: D-ReLU top-k   (Section 3.1, threshold and piecewise equations)
# ---------------------------------------------------------------------------

def test_topk_bruteforce_random_and_quantised():
    rng = np.random.default_rng(1)
    for D, k in [(8, 3), (16, 16), (16, 1), (33, 7), (64, 16), (128, 32)]:
        X = rng.standard_normal((40, D)).astype(np.float32)
        Xq = np.round(rng.standard_normal((40, D)) * 2).astype(np.float32)  # many ties
        for A in (X, Xq):
            vals, idx = oracle.topk(A, k)
            for i in range(A.shape[0]):
                keep = brute_topk_row(A[i], k)
                assert idx[i].tolist() == keep
                assert np.array_equal(vals[i], A[i, keep].astype(np.float64))


def test_topk_invariants():
    rng = np.random.default_rng(2)
    X = np.round(rng.standard_normal((200, 64)) * 3).astype(np.float32) / 3
    k = 16
    vals, idx = oracle.topk(X, k)
    assert idx.shape == (200, k)
    assert np.all(np.diff(idx, axis=1) > 0)                    # strictly ascending, hence exactly k distinct
    for i in range(X.shape[0]):
        kept = np.zeros(64, dtype=bool)
        kept[idx[i]] = True
        th = vals[i].min()
        assert np.all(X[i, ~kept] <= th)                       # every dropped value <= every kept value
        tie_dropped = np.nonzero(~kept & (X[i] == th))[0]
        tie_kept = np.nonzero(kept & (X[i] == th))[0]
        if tie_dropped.size:
            assert tie_dropped.min() > tie_kept.max()          # ties resolved to the lowest columns


def test_topk_special_cases():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((50, 32)).astype(np.float32)
    X[7, 5] = X[7, 20] = X[7].max() + 1                         # duplicated maximum: first occurrence wins
    vals, idx = oracle.topk(X, 1)
    assert np.array_equal(idx[:, 0], np.argmax(X, axis=1))
    assert idx[7, 0] == 5
    vals, idx = oracle.topk(X, 32)                              # k = D is the identity
    assert np.array_equal(idx, np.tile(np.arange(32), (50, 1)))
    assert np.array_equal(vals, X.astype(np.float64))
    assert np.array_equal(oracle.densify(vals, idx, 32), X.astype(np.float64))


def test_topk_constructed_ties_and_signed_zero():
    D, k = 16, 5
    allsame = np.full((1, D), 2.5, np.float32)
    _, idx = oracle.topk(allsame, k)
    assert idx[0].tolist() == [0, 1, 2, 3, 4]
    row = np.array([[1, 9, 3, 3, 9, 3, 0, 3, -1, 3, 9, 2, 3, 3, 3, 3]], np.float32)
    _, idx = oracle.topk(row, k)                               # three 9s, then the two left-most 3s
    assert idx[0].tolist() == [1, 2, 3, 4, 10]
    z = np.array([[-1, -0.0, 0.0, -2, 0.0, -0.0, -3, -4]], np.float32)
    vals, idx = oracle.topk(z, 3)                              # -0.0 == +0.0: columns 1, 2, 4
    assert idx[0].tolist() == [1, 2, 4]
    assert np.signbit(vals[0, 0]) and not np.signbit(vals[0, 1])   # values are copied, sign of zero kept
    neg = -np.arange(1, 9, dtype=np.float32)[None, :]          # all negative: still the k largest, not clamped
    vals, idx = oracle.topk(neg, 2)
    assert idx[0].tolist() == [0, 1] and vals[0].tolist() == [-1.0, -2.0]


def test_topk_rejects_bad_arguments():
    X = np.zeros((2, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.topk(X, 5)
    with pytest.raises(ValueError):
        oracle.topk(X, 0)
    X[1, 2] = np.nan
    with pytest.raises(ValueError):
        oracle.topk(X, 2)


def test_topk_matches_library_selection_on_tie_free_rows():
    import torch
    rng = np.random.default_rng(4)
    X = rng.standard_normal((300, 128)).astype(np.float32)
    k = 32
    vals, idx = oracle.topk(X, k)
    part = np.sort(np.argpartition(-X, k - 1, axis=1)[:, :k], axis=1)
    assert np.array_equal(idx, part)
    tv, ti = torch.topk(torch.from_numpy(X), k, dim=1)
    assert np.array_equal(idx, np.sort(ti.numpy(), axis=1))
    assert np.allclose(np.sort(vals, axis=1), np.sort(tv.numpy().astype(np.float64), axis=1), rtol=0, atol=0)


def test_topk_golden_hand_worked_rows():
    """Rows worked by hand from the D-ReLU definition (file header carries the derivation)."""
    rows, expect = [], []
    with open(os.path.join(GOLDEN, "drelu_rows.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            k, xs, keep = line.split("|")
            rows.append((int(k), np.array([float(v) for v in xs.split()], np.float32)))
            expect.append([int(v) for v in keep.split()])
    for (k, x), keep in zip(rows, expect):
        vals, idx = oracle.topk(x[None, :], k)
        assert idx[0].tolist() == keep
        assert vals[0].tolist() == [float(x[c]) for c in keep]


# ---------------------------------------------------------------------------
# O2: edge values of the modules
# ---------------------------------------------------------------------------

def test_normalize_mean_and_sym_against_scipy():
    rng = np.random.default_rng(5)
    M, N = 37, 23
    rowptr, colidx, _ = random_csr(rng, M, N, 9, dup=True)
    ones = np.ones(colidx.shape[0])
    A = sp.csr_matrix((ones, colidx, rowptr), shape=(M, N))   # keeps duplicates as separate stored entries
    deg_in = np.diff(rowptr)
    deg_out = np.bincount(colidx, minlength=N)
    mean = oracle.csr_normalize(oracle.NORM_MEAN, M, N, rowptr, colidx)
    sym = oracle.csr_normalize(oracle.NORM_SYM, M, N, rowptr, colidx)
    rows = np.repeat(np.arange(M), deg_in)
    assert np.array_equal(mean, (1.0 / deg_in[rows]).astype(np.float32))
    expect = 1.0 / np.sqrt(np.maximum(deg_in[rows], 1) * np.maximum(deg_out[colidx], 1).astype(np.float64))
    assert np.array_equal(sym, expect.astype(np.float32))
    # mean-normalised rows sum to one (non-empty rows), via scipy
    Am = sp.csr_matrix((mean.astype(np.float64), colidx, rowptr), shape=(M, N))
    s = np.asarray(Am.sum(axis=1)).ravel()
    assert np.allclose(s[deg_in > 0], 1.0, atol=1e-6) and np.all(s[deg_in == 0] == 0)
    # D_in^-1/2 A D_out^-1/2 via scipy diagonal scaling
    Din = sp.diags(1.0 / np.sqrt(np.maximum(deg_in, 1)))
    Dout = sp.diags(1.0 / np.sqrt(np.maximum(deg_out, 1)))
    ref = (Din @ A @ Dout).toarray()
    assert np.allclose(dense_of(rowptr, colidx, sym, M, N), ref, atol=1e-6)


# ---------------------------------------------------------------------------
# O3: forward SpMM on the row-sparse operand
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("dup", [False, True])
def test_spmm_fwd_dense_and_scipy(dup):
    rng = np.random.default_rng(6)
    M, N, D, k = 29, 31, 16, 5
    rowptr, colidx, avals = random_csr(rng, M, N, 7, dup=dup)
    X = rng.standard_normal((N, D)).astype(np.float32)
    vals, idx = oracle.topk(X, k)
    H, l1row, l1elem = oracle.spmm_fwd(rowptr, colidx, avals, vals, idx, D, want_l1elem=True)
    # dense definition with an independently built f(X): keep the k largest per row by sorting
    fX = np.zeros((N, D))
    for j in range(N):
        keep = brute_topk_row(X[j], k)
        fX[j, keep] = X[j, keep]
    A = dense_of(rowptr, colidx, avals, M, N)
    assert np.allclose(H, A @ fX, rtol=1e-13, atol=1e-13)
    As = sp.csr_matrix((avals.astype(np.float64), colidx, rowptr), shape=(M, N))
    assert np.allclose(H, As @ fX, rtol=1e-13, atol=1e-13)
    assert np.allclose(l1elem, A @ np.abs(fX), rtol=1e-13, atol=1e-13)
    assert np.allclose(l1row, l1elem.sum(axis=1), rtol=1e-12)
    empty = np.diff(rowptr) == 0
    assert empty.any() and np.all(H[empty] == 0.0)


def test_spmm_fwd_k_equals_D_is_textbook_spmm():
    rng = np.random.default_rng(7)
    M, N, D = 20, 25, 12
    rowptr, colidx, avals = random_csr(rng, M, N, 6)
    X = rng.standard_normal((N, D))
    vals, idx = oracle.topk(X, D)
    H, _ = oracle.spmm_fwd(rowptr, colidx, avals, vals, idx, D)
    assert np.allclose(H, dense_of(rowptr, colidx, avals, M, N) @ X, rtol=1e-13, atol=1e-13)


def test_spmm_fwd_mean_of_constant_and_linearity():
    rng = np.random.default_rng(8)
    M, N, D, k = 30, 30, 8, 3
    rowptr, colidx, _ = random_csr(rng, M, N, 6)
    mean = oracle.csr_normalize(oracle.NORM_MEAN, M, N, rowptr, colidx)
    row = rng.standard_normal(D)
    X = np.tile(row, (N, 1))                                    # every source row identical
    vals, idx = oracle.topk(X, k)
    H, _ = oracle.spmm_fwd(rowptr, colidx, mean, vals, idx, D)
    fx = oracle.densify(vals[:1], idx[:1], D)[0]
    nonempty = np.diff(rowptr) > 0
    assert np.allclose(H[nonempty], fx[None, :], atol=1e-6)     # mean of identical rows is that row
    # linearity in the CBSR values (indices held fixed)
    v2 = rng.standard_normal(vals.shape)
    H1, _ = oracle.spmm_fwd(rowptr, colidx, mean, vals, idx, D)
    H2, _ = oracle.spmm_fwd(rowptr, colidx, mean, v2, idx, D)
    H3, _ = oracle.spmm_fwd(rowptr, colidx, mean, 2.0 * vals - 3.0 * v2, idx, D)
    assert np.allclose(H3, 2.0 * H1 - 3.0 * H2, atol=1e-12)


# ---------------------------------------------------------------------------
# O5: stable transpose
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("dup", [False, True])
def test_transpose_bruteforce(dup):
    rng = np.random.default_rng(9)
    M, N = 41, 17
    rowptr, colidx, vals = random_csr(rng, M, N, 8, dup=dup)
    t_rowptr, t_colidx, t_vals = oracle.csr_transpose(M, N, rowptr, colidx, vals)
    triples = []
    for i in range(M):
        for pos in range(rowptr[i], rowptr[i + 1]):
            triples.append((int(colidx[pos]), i, pos))
    triples.sort()                                              # by column, then original row, then storage position
    assert t_rowptr.tolist() == [0] + np.cumsum(np.bincount(colidx, minlength=N)).tolist()
    assert t_colidx.tolist() == [t[1] for t in triples]
    assert np.array_equal(t_vals, vals[[t[2] for t in triples]])


def test_transpose_involution_and_scipy():
    rng = np.random.default_rng(10)
    M, N = 33, 47
    rowptr, colidx, vals = random_csr(rng, M, N, 9)
    # sort columns inside rows first so that the double transpose must reproduce the input exactly
    for i in range(M):
        s = slice(rowptr[i], rowptr[i + 1])
        o = np.argsort(colidx[s], kind="stable")
        colidx[s], vals[s] = colidx[s][o], vals[s][o]
    t = oracle.csr_transpose(M, N, rowptr, colidx, vals)
    tt = oracle.csr_transpose(N, M, *t)
    assert np.array_equal(tt[0], rowptr) and np.array_equal(tt[1], colidx) and np.array_equal(tt[2], vals)
    ref = sp.csr_matrix((vals, colidx, rowptr), shape=(M, N)).T.tocsr()
    ref.sort_indices()
    assert np.array_equal(t[0], ref.indptr) and np.array_equal(t[1], ref.indices) and np.array_equal(t[2], ref.data)


def test_generator_pinned_is_transpose_of_pins(tiny_graph):
    g = tiny_graph
    t_rowptr, t_colidx, _ = oracle.csr_transpose(g.pins.n_rows, g.pins.n_cols, g.pins.rowptr, g.pins.colidx)
    assert np.array_equal(t_rowptr, g.pinned.rowptr) and np.array_equal(t_colidx, g.pinned.colidx)
    p2 = transpose_pattern(g.pinned)
    assert np.array_equal(p2.rowptr, g.pins.rowptr) and np.array_equal(p2.colidx, g.pins.colidx)


# ---------------------------------------------------------------------------
# O6: backward SpMM gated by the saved indices
# ---------------------------------------------------------------------------

def test_spmm_bwd_dense_formula_and_adjoint():
    rng = np.random.default_rng(11)
    M, N, D, k = 26, 19, 16, 6
    rowptr, colidx, avals = random_csr(rng, M, N, 7, dup=True)
    X = rng.standard_normal((N, D)).astype(np.float32)
    vals, idx = oracle.topk(X, k)
    dH = rng.standard_normal((M, D))
    t = oracle.csr_transpose(M, N, rowptr, colidx, avals)
    G, l1row, l1elem = oracle.spmm_bwd(*t, dH, idx, want_l1elem=True)
    A = dense_of(rowptr, colidx, avals, M, N)
    full = A.T @ dH                                              # dense dL/dX before gating
    assert np.allclose(G, np.take_along_axis(full, idx.astype(np.int64), axis=1), rtol=1e-13, atol=1e-13)
    assert np.allclose(l1elem, np.take_along_axis(A.T @ np.abs(dH), idx.astype(np.int64), axis=1), rtol=1e-12)
    assert np.allclose(l1row, l1elem.sum(axis=1), rtol=1e-12)
    # adjoint identity <A f(X), R> = <vals, G(R)>
    H, _ = oracle.spmm_fwd(rowptr, colidx, avals, vals, idx, D)
    assert np.isclose(np.sum(H * dH), np.sum(vals * G), rtol=1e-12)


# ---------------------------------------------------------------------------
# the layer: dense re-formulation, autograd, finite differences
# ---------------------------------------------------------------------------

def _small_layer(seed=0, Nc=48, Nn=30, D=16, kc=5, kn=4):
    rng = np.random.default_rng(seed)
    g = make_graph("tiny", seed=seed, Nc=Nc, Nn=Nn, grid=(8, 6))
    near = oracle.relation(g.near, oracle.NORM_MEAN)
    pins = oracle.relation(g.pins, oracle.NORM_MEAN)
    pinned = oracle.relation(g.pinned, oracle.NORM_SYM)
    T = make_tensors(Nc, Nn, D, seed=seed)
    return g, near, pins, pinned, T, rng, kc, kn


def _dense_layer_numpy(near, pins, pinned, Xc, Xn, W, kc, kn):
    def f(X, k):
        out = np.zeros_like(X)
        for j in range(X.shape[0]):
            keep = brute_topk_row(X[j], k)
            out[j, keep] = X[j, keep]
        return out
    An = dense_of(near.rowptr, near.colidx, near.vals, near.M, near.N)
    Ap = dense_of(pins.rowptr, pins.colidx, pins.vals, pins.M, pins.N)
    Aq = dense_of(pinned.rowptr, pinned.colidx, pinned.vals, pinned.M, pinned.N)
    Xsc, Xsn = f(Xc, kc), f(Xn, kn)
    Zn = Xsc @ W["self_near"] + (An @ Xsc) @ W["neigh_near"]
    Yn = Xsn @ W["self_pins"] + (Ap @ Xsc) @ W["neigh_pins"]
    Zq = (Aq @ Xsn) @ W["pinned"]
    return np.maximum(Zn, Zq), Yn, (Zn >= Zq), (An, Ap, Aq, Xsc, Xsn)


def test_heteroconv_fwd_dense_reformulation():
    g, near, pins, pinned, T, rng, kc, kn = _small_layer()
    Xc, Xn = T.X_cell.astype(np.float64), T.X_net.astype(np.float64)
    W = {n: w.astype(np.float64) for n, w in T.W.items()}
    o = oracle.heteroconv_fwd(near, pins, pinned, Xc, Xn, W, kc, kn)
    Yc, Yn, M, (An, Ap, Aq, Xsc, Xsn) = _dense_layer_numpy(near, pins, pinned, Xc, Xn, W, kc, kn)
    assert np.allclose(o["Y_cell"], Yc, rtol=1e-12, atol=1e-12)
    assert np.allclose(o["Y_net"], Yn, rtol=1e-12, atol=1e-12)
    assert np.array_equal(o["mask"].astype(bool), M)
    assert np.allclose(o["H_near"], An @ Xsc, atol=1e-12)
    assert np.allclose(o["H_pins"], Ap @ Xsc, atol=1e-12)
    assert np.allclose(o["H_pinned"], Aq @ Xsn, atol=1e-12)
    # both branches feed the cell output somewhere (otherwise the max-merge is untested)
    assert 0 < o["mask"].mean() < 1
    # the per-element L1 bound dominates the magnitude of every output
    assert np.all(np.abs(o["Y_cell"]) <= o["l1_cell"] * (1 + 1e-12) + 1e-300)
    assert np.all(np.abs(o["Y_net"]) <= o["l1_net"] * (1 + 1e-12) + 1e-300)


def test_heteroconv_bwd_matches_torch_autograd_on_dense_form():
    import torch
    g, near, pins, pinned, T, rng, kc, kn = _small_layer(seed=3)
    Xc, Xn = T.X_cell.astype(np.float64), T.X_net.astype(np.float64)
    W = {n: w.astype(np.float64) for n, w in T.W.items()}
    dYc, dYn = T.dY_cell.astype(np.float64), T.dY_net.astype(np.float64)
    o = oracle.heteroconv_fwd(near, pins, pinned, Xc, Xn, W, kc, kn)
    b = oracle.heteroconv_bwd(near, pins, pinned, W, o, dYc, dYn)

    # dense graph of torch ops with the D-ReLU selection held fixed as 0/1 masks and torch's own max
    _, _, _, (An, Ap, Aq, Xsc, Xsn) = _dense_layer_numpy(near, pins, pinned, Xc, Xn, W, kc, kn)
    tXc = torch.tensor(Xc, requires_grad=True)
    tXn = torch.tensor(Xn, requires_grad=True)
    tW = {n: torch.tensor(w, requires_grad=True) for n, w in W.items()}
    mc, mn = torch.tensor((Xsc != 0) | (Xsc == Xc)), torch.tensor((Xsn != 0) | (Xsn == Xn))
    sel_c = torch.zeros_like(tXc, dtype=torch.bool)
    sel_c.scatter_(1, torch.tensor(o["idx_cell"].astype(np.int64)), True)
    sel_n = torch.zeros_like(tXn, dtype=torch.bool)
    sel_n.scatter_(1, torch.tensor(o["idx_net"].astype(np.int64)), True)
    fc, fn = tXc * sel_c, tXn * sel_n
    tAn, tAp, tAq = torch.tensor(An), torch.tensor(Ap), torch.tensor(Aq)
    Zn = fc @ tW["self_near"] + (tAn @ fc) @ tW["neigh_near"]
    Yn = fn @ tW["self_pins"] + (tAp @ fc) @ tW["neigh_pins"]
    Zq = (tAq @ fn) @ tW["pinned"]
    Yc = torch.maximum(Zn, Zq)
    loss = (Yc * torch.tensor(dYc)).sum() + (Yn * torch.tensor(dYn)).sum()
    loss.backward()
    assert np.allclose(b["dX_cell"], tXc.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(b["dX_net"], tXn.grad.numpy(), rtol=1e-10, atol=1e-12)
    for n in oracle.WEIGHT_NAMES:
        assert np.allclose(b["dW"][n], tW[n].grad.numpy(), rtol=1e-10, atol=1e-12), n
    # compact and dense forms agree, dense is zero off the saved positions
    assert np.array_equal(np.take_along_axis(b["dX_cell"], o["idx_cell"].astype(np.int64), 1), b["dXs_cell"])
    assert np.count_nonzero(b["dX_cell"]) <= o["idx_cell"].size
    assert np.count_nonzero(b["dX_net"]) <= o["idx_net"].size


def test_heteroconv_bwd_finite_differences():
    """Central differences in fp64 on L = <Y_cell, R_cell> + <Y_net, R_net>.  The layer is piecewise
    linear in X and bilinear in (X, W); away from top-k and max ties the FD quotient is exact up to
    rounding.  Probed entries are restricted to rows whose selection margins exceed 10 eps."""
    g, near, pins, pinned, T, rng, kc, kn = _small_layer(seed=5)
    Xc, Xn = T.X_cell.astype(np.float64), T.X_net.astype(np.float64)
    W = {n: w.astype(np.float64) for n, w in T.W.items()}
    Rc, Rn = T.dY_cell.astype(np.float64), T.dY_net.astype(np.float64)
    eps = 1e-6

    def loss(Xc_, Xn_, W_):
        o_ = oracle.heteroconv_fwd(near, pins, pinned, Xc_, Xn_, W_, kc, kn)
        return float(np.sum(o_["Y_cell"] * Rc) + np.sum(o_["Y_net"] * Rn)), o_

    L0, o = loss(Xc, Xn, W)
    b = oracle.heteroconv_bwd(near, pins, pinned, W, o, Rc, Rn)
    assert np.min(np.abs(o["Z_near"] - o["Z_pinned"])) > 1e-3   # max-merge margins are wide on this input

    def margin(X, k):
        s = -np.sort(-X, axis=1)
        return s[:, k - 1] - s[:, k]
    assert margin(Xc, kc).min() > 100 * eps and margin(Xn, kn).min() > 100 * eps

    checked = 0
    for name, X, grad in (("cell", Xc, b["dX_cell"]), ("net", Xn, b["dX_net"])):
        for _ in range(25):
            j, c = int(rng.integers(X.shape[0])), int(rng.integers(X.shape[1]))
            Xp, Xm = X.copy(), X.copy()
            Xp[j, c] += eps
            Xm[j, c] -= eps
            if name == "cell":
                fd = (loss(Xp, Xn, W)[0] - loss(Xm, Xn, W)[0]) / (2 * eps)
            else:
                fd = (loss(Xc, Xp, W)[0] - loss(Xc, Xm, W)[0]) / (2 * eps)
            assert abs(fd - grad[j, c]) <= 1e-6 * max(1.0, abs(grad[j, c])), (name, j, c, fd, grad[j, c])
            checked += 1
    for n in oracle.WEIGHT_NAMES:
        for _ in range(6):
            r, c = int(rng.integers(W[n].shape[0])), int(rng.integers(W[n].shape[1]))
            Wp = {m: w.copy() for m, w in W.items()}
            Wm = {m: w.copy() for m, w in W.items()}
            Wp[n][r, c] += eps
            Wm[n][r, c] -= eps
            fd = (loss(Xc, Xn, Wp)[0] - loss(Xc, Xn, Wm)[0]) / (2 * eps)
            assert abs(fd - b["dW"][n][r, c]) <= 1e-6 * max(1.0, abs(b["dW"][n][r, c])), (n, r, c)
            checked += 1
    assert checked == 80


def test_heteroconv_on_tiny_workload_runs_and_is_consistent(tiny_graph, tiny_tensors):
    g, T = tiny_graph, tiny_tensors
    near = oracle.relation(g.near, oracle.NORM_MEAN)
    pins = oracle.relation(g.pins, oracle.NORM_MEAN)
    pinned = oracle.relation(g.pinned, oracle.NORM_SYM)
    o = oracle.heteroconv_fwd(near, pins, pinned, T.X_cell, T.X_net, T.W, 16, 16)
    assert np.all(np.diff(o["idx_cell"], axis=1) > 0) and o["idx_cell"].shape == (g.Nc, 16)
    # adjoint identity through the whole layer: <Y(R-weighted)> reproduced by <X, dX> because the layer is
    # positively homogeneous of degree 1 in (X_cell, X_net) jointly (top-k, max and the linear maps all are)
    b = oracle.heteroconv_bwd(near, pins, pinned, T.W, o, T.dY_cell, T.dY_net)
    lhs = np.sum(o["Y_cell"] * T.dY_cell) + np.sum(o["Y_net"] * T.dY_net)
    rhs = np.sum(T.X_cell.astype(np.float64) * b["dX_cell"]) + np.sum(T.X_net.astype(np.float64) * b["dX_net"])
    assert np.isclose(lhs, rhs, rtol=1e-10)
