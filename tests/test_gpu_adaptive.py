"""Degree-adaptive K through the C ABI (dr_topk_ranked, dr_spmm_fwd_adaptive, dr_spmm_bwd_adaptive) against the
fp64 oracle (oracle/adaptive.py): rank-ordered selections bit for bit, SpMM results element by element, and a
sampled check on the 1.2 M-cell graph in the configuration the measurements use."""
import numpy as np
import pytest
import torch

import oracle
from oracle import adaptive as oad
import paper_2508_16769_amd as P
from circuit_synth import make_graph, workload
from gpu_util import assert_elem_bound, assert_row_bound, dev, host_idx, random_csr, say
from sampled_checks import sub_rows

pytestmark = pytest.mark.gpu


def gpu_topk_ranked(X, k):
    n, D = X.shape
    vals = torch.full((n, k), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((n, k), -1, dtype=torch.int16, device="cuda")
    P.dr_topk_ranked(dev(X), k, vals, idx)
    torch.cuda.synchronize()
    return vals, idx


@pytest.mark.parametrize("n,D,k", [(1000, 128, 32), (777, 64, 16), (513, 128, 64), (300, 96, 5), (64, 1024, 300),
                                   (100, 5, 1), (257, 128, 128), (400, 256, 9)])
def test_topk_ranked_bit_exact(n, D, k):
    say(f"dr_topk_ranked n={n} D={D} k={k}")
    rng = np.random.default_rng(n + D + k)
    X = rng.standard_normal((n, D)).astype(np.float32)
    X[1] = 0.25                                            # one value everywhere: ties cut by column
    X[2, ::2] = -0.0
    X[2, 1::2] = 0.0                                       # signed zeros compare equal
    X[3] = -np.abs(X[3])                                   # all negative
    X[4, : D // 2] = X[4, D // 2: 2 * (D // 2)]            # every value twice
    m = min(n - 5, n // 4)
    X[5: 5 + m] = rng.integers(0, 8, size=(m, D)).astype(np.float32)   # heavy ties
    vals, idx = gpu_topk_ranked(X, k)
    ov, oi = oad.topk_ranked(X, k)
    assert np.array_equal(host_idx(idx), oi)
    assert np.array_equal(vals.cpu().numpy().view(np.uint32), ov.astype(np.float32).view(np.uint32))
    # the same selection as dr_topk, which lists it by column
    v2 = torch.empty((n, k), dtype=torch.float32, device="cuda")
    i2 = torch.empty((n, k), dtype=torch.int16, device="cuda")
    P.dr_topk(dev(X), k, v2, i2)
    torch.cuda.synchronize()
    assert np.array_equal(np.sort(host_idx(idx), axis=1), host_idx(i2))


# M, N, max_deg, D, (t1, t2, k1, k2, k3), dup, evil
CASES = [
    (1000, 900, 12, 128, (4, 8, 32, 16, 8), True, True),
    (777, 1301, 9, 128, (3, 6, 16, 4, 2), False, True),
    (600, 500, 10, 64, (2, 5, 8, 8, 1), True, True),
    (600, 500, 10, 96, (0, 4, 24, 7, 3), False, True),       # t1 = 0: only empty rows are "low"
    (515, 400, 20, 128, (5, 10, 64, 32, 16), True, True),    # the widest supported k1
    (300, 200, 7, 64, (3, 3, 5, 5, 2), True, False),         # two classes
    (300, 300, 7, 32, (100, 200, 32, 2, 1), False, False),   # everything in the low class, k1 = D
    (100, 80, 5, 5, (1, 2, 3, 2, 1), True, False),
]


def _ids():
    return [f"M{c[0]}_D{c[3]}_k{'-'.join(map(str, c[4][2:]))}" for c in CASES]


def _inputs(case, seed):
    M, N, max_deg, D, cls, dup, evil = case
    rng = np.random.default_rng(seed)
    rowptr, colidx, avals = random_csr(rng, M, N, max_deg, dup=dup, evil_rows=(5, M // 2) if evil else (),
                                       evil_deg=min(700, 3 * N) if dup else min(N, 300))
    X = rng.standard_normal((N, D)).astype(np.float32)
    return rowptr, colidx, avals, X, oad.DegreeClasses(*cls), rng


def _edge_classes(At, A, cls, rowptr):
    """dr_degree_edge_classes, checked bit for bit: class of the destination of every entry of A^T."""
    ecls = torch.full((At.nnz,), 255, dtype=torch.uint8, device="cuda")
    P.dr_degree_edge_classes(At, A.rowptr, tuple(cls), ecls)
    torch.cuda.synchronize()
    deg = np.diff(np.asarray(rowptr))
    want = np.where(deg <= cls.t1, 0, np.where(deg <= cls.t2, 1, 2))[At.colidx.cpu().numpy()]
    assert np.array_equal(ecls.cpu().numpy(), want.astype(np.uint8))
    return ecls


@pytest.mark.parametrize("case", CASES, ids=_ids())
def test_spmm_fwd_adaptive_parity(case):
    M, N, _, D, _, _, _ = case
    rowptr, colidx, avals, X, cls, rng = _inputs(case, 11)
    say(f"dr_spmm_fwd_adaptive M={M} N={N} D={D} classes={tuple(cls)}")
    ov, oi = oad.topk_ranked(X, cls.k1)
    H_o, L1 = oad.spmm_fwd_adaptive(rowptr, colidx, avals, ov, oi, D, cls)
    vals, idx = gpu_topk_ranked(X, cls.k1)
    A = P.Csr(M, N, dev(rowptr), dev(colidx), dev(avals))
    H = torch.full((M, D), float("nan"), dtype=torch.float32, device="cuda")
    P.dr_spmm_fwd_adaptive(A, vals, idx, D, tuple(cls), H)
    torch.cuda.synchronize()
    got = H.cpu().numpy()
    assert_row_bound(got, H_o, L1.sum(axis=1), "H")
    assert_elem_bound(got, H_o, L1, "H")


@pytest.mark.parametrize("case", CASES, ids=_ids())
def test_spmm_bwd_adaptive_parity(case):
    M, N, _, D, _, _, _ = case
    rowptr, colidx, avals, X, cls, rng = _inputs(case, 12)
    say(f"dr_spmm_bwd_adaptive M={M} N={N} D={D} classes={tuple(cls)}")
    ov, oi = oad.topk_ranked(X, cls.k1)
    dH = rng.standard_normal((M, D)).astype(np.float32)
    G_o, L1 = oad.spmm_bwd_adaptive(rowptr, colidx, avals, dH, oi, N, cls)
    _, idx = gpu_topk_ranked(X, cls.k1)
    A = P.Csr(M, N, dev(rowptr), dev(colidx), dev(avals))
    At = P.device_transpose(A)
    G = torch.full((N, cls.k1), float("nan"), dtype=torch.float32, device="cuda")
    ecls = _edge_classes(At, A, cls, rowptr)
    P.dr_spmm_bwd_adaptive(At, ecls, dev(dH), idx, D, tuple(cls), G)
    torch.cuda.synchronize()
    got = G.cpu().numpy()
    assert_row_bound(got, G_o, L1.sum(axis=1), "G")
    assert_elem_bound(got, G_o, L1, "G")
    # accumulate adds to what is there
    P.dr_spmm_bwd_adaptive(At, ecls, dev(dH), idx, D, tuple(cls), G, accumulate=True)
    torch.cuda.synchronize()
    assert_row_bound(G.cpu().numpy(), 2 * G_o, 2 * L1.sum(axis=1), "G accumulated")


def test_equal_widths_reproduce_the_uniform_kernels():
    """k1 = k2 = k3: the adaptive kernels compute the uniform DR-SpMM (checked against dr_spmm_fwd / dr_spmm_bwd on the
    column-ordered CBSR of the same selection): every output element receives the same terms in the same edge order
    on both paths -- the pairs of one source row have distinct columns -- so the results agree bit for bit."""
    case = (1000, 900, 12, 128, (4, 8, 16, 16, 16), True, True)
    M, N, _, D, _, _, _ = case
    rowptr, colidx, avals, X, cls, rng = _inputs(case, 13)
    say("adaptive kernels with equal widths vs the uniform kernels")
    k = cls.k1
    vr, ir = gpu_topk_ranked(X, k)
    vc = torch.empty((N, k), dtype=torch.float32, device="cuda")
    ic = torch.empty((N, k), dtype=torch.int16, device="cuda")
    P.dr_topk(dev(X), k, vc, ic)
    A = P.Csr(M, N, dev(rowptr), dev(colidx), dev(avals))
    At = P.device_transpose(A)
    Ha = torch.empty((M, D), dtype=torch.float32, device="cuda")
    Hu = torch.empty_like(Ha)
    P.dr_spmm_fwd_adaptive(A, vr, ir, D, tuple(cls), Ha)
    P.dr_spmm_fwd(A, vc, ic, D, k, Hu)
    dH = dev(rng.standard_normal((M, D)).astype(np.float32))
    Ga = torch.empty((N, k), dtype=torch.float32, device="cuda")
    Gu = torch.empty_like(Ga)
    ecls = _edge_classes(At, A, cls, rowptr)
    P.dr_spmm_bwd_adaptive(At, ecls, dH, ir, D, tuple(cls), Ga)
    P.dr_spmm_bwd(At, dH, ic, D, k, Gu)
    torch.cuda.synchronize()
    assert torch.equal(Ha, Hu)          # distinct columns of a source row: each output element sees the same terms in the same order
    pos = np.argsort(host_idx(ir), axis=1, kind="stable")
    assert np.array_equal(np.take_along_axis(Ga.cpu().numpy(), pos, axis=1), Gu.cpu().numpy())


def test_adaptive_argument_errors():
    say("adaptive argument errors")
    rng = np.random.default_rng(0)
    rowptr, colidx, avals = random_csr(rng, 50, 40, 5)
    A = P.Csr(50, 40, dev(rowptr), dev(colidx), dev(avals))
    v = torch.zeros((40, 8), dtype=torch.float32, device="cuda")
    i = torch.zeros((40, 8), dtype=torch.int16, device="cuda")
    H = torch.zeros((50, 64), dtype=torch.float32, device="cuda")
    for bad in ((3, 2, 8, 4, 2), (-1, 2, 8, 4, 2), (1, 2, 4, 8, 2), (1, 2, 8, 4, 0), (1, 2, 65, 4, 2)):
        with pytest.raises(P.DrError) as e:
            P.dr_spmm_fwd_adaptive(A, v, i, 64, bad, H)
        assert e.value.code in (P.DR_ERR_INVALID_ARG, P.DR_ERR_UNSUPPORTED), bad
    with pytest.raises(P.DrError):
        P.dr_spmm_fwd_adaptive(A, v, i, 128, (1, 2, 96, 4, 2), H)       # k1 above 64
    with pytest.raises(P.DrError):
        P.dr_topk_ranked(torch.zeros((4, 8), device="cuda"), 9, v, i)


def test_adaptive_on_the_large_graph_sampled():
    """The 1.2 M-cell `near` relation (power-law in-degrees) with three degree classes: the kernels run on the whole
    graph, the oracle recomputes sampled destination rows (forward) and source rows (backward) one by one."""
    w = workload("large")
    D = w["D"]
    cls = oad.DegreeClasses(8, 32, 32, 16, 8)
    say("large: generating graph")
    g = make_graph("large", seed=0)
    rel = oracle.relation(g.near, oracle.NORM_MEAN)
    rng = np.random.default_rng(99)
    X = rng.standard_normal((g.Nc, D)).astype(np.float32)
    dH = rng.standard_normal((g.Nc, D)).astype(np.float32)
    A = P.device_relation(g.near, P.DR_NORM_MEAN)
    At = P.device_transpose(A)
    say("large: kernels")
    vals, idx = gpu_topk_ranked(X, cls.k1)
    H = torch.empty((g.Nc, D), dtype=torch.float32, device="cuda")
    G = torch.empty((g.Nc, cls.k1), dtype=torch.float32, device="cuda")
    P.dr_spmm_fwd_adaptive(A, vals, idx, D, tuple(cls), H)
    ecls = _edge_classes(At, A, cls, rel.rowptr)
    P.dr_spmm_bwd_adaptive(At, ecls, dev(dH), idx, D, tuple(cls), G)
    torch.cuda.synchronize()
    deg = np.diff(rel.rowptr)
    assert (deg <= cls.t1).any() and ((deg > cls.t1) & (deg <= cls.t2)).any() and (deg > cls.t2).any()
    # ---- selections on sampled rows ----
    rows = np.sort(rng.choice(g.Nc, 2000, replace=False))
    ov, oi = oad.topk_ranked(X[rows], cls.k1)
    sel = torch.from_numpy(rows).cuda()
    assert np.array_equal(host_idx(idx[sel]), oi)
    assert np.array_equal(vals[sel].cpu().numpy().astype(np.float64), ov)
    # ---- forward: sampled destinations of every class, with all their edges ----
    pick = np.concatenate([rng.choice(np.where(m)[0], 120, replace=False)
                           for m in (deg <= cls.t1, (deg > cls.t1) & (deg <= cls.t2), deg > cls.t2)])
    pick = np.sort(pick)
    say(f"large: forward on {len(pick)} sampled destinations (max degree {deg[pick].max()})")
    sub_rp, local, a, uniq = sub_rows(rel, pick)
    sv, si = oad.topk_ranked(X[uniq], cls.k1)
    H_o, L1 = oad.spmm_fwd_adaptive(sub_rp, local, a, sv, si, D, cls)
    got = H[torch.from_numpy(pick).cuda()].cpu().numpy()
    assert_row_bound(got, H_o, L1.sum(axis=1), "H large")
    assert_elem_bound(got, H_o, L1, "H large")
    # ---- backward: sampled sources; their edges are the rows of A^T, whose class is that of the edge's destination ----
    t_rp, t_ci, t_v = oracle.csr_transpose(rel.M, rel.N, rel.rowptr, rel.colidx, rel.vals)
    srcs = np.sort(rng.choice(g.Nc, 300, replace=False))
    say(f"large: backward on {len(srcs)} sampled sources")
    _, oi_s = oad.topk_ranked(X[srcs], cls.k1)
    Gs = G[torch.from_numpy(srcs).cuda()].cpu().numpy()
    k_of = cls.k_of_degree(deg)
    for n_, j in enumerate(srcs):
        e = np.arange(t_rp[j], t_rp[j + 1])
        dst = t_ci[e]
        terms = t_v[e].astype(np.float64)[:, None] * dH[dst][:, oi_s[n_]].astype(np.float64)     # [edges, k1]
        terms = terms * (k_of[dst][:, None] > np.arange(cls.k1)[None, :])
        want, l1 = terms.sum(axis=0), np.abs(terms).sum(axis=0)
        assert np.all(np.abs(Gs[n_] - want) <= 1e-5 * l1 + 1e-30), j
        assert np.all(Gs[n_][l1 == 0] == 0), j
