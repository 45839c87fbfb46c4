"""GPU parity: every C-ABI entry point against the CPU oracle, element by element, on seeded inputs
that span several tiles and ragged tails.  Integer / index results are bit-exact; fp32 results are
within 1e-4 x (row L1 norm of the contributing terms), plus a stricter per-element bound."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_16769_amd as P
from circuit_synth import make_graph, make_tensors, workload
from gpu_util import (HostPattern, assert_elem_bound, assert_row_bound, cells_with_agreeing_masks, dev, host_idx, random_csr,
                      say)

pytestmark = pytest.mark.gpu


def gpu_topk(X, k):
    n, D = X.shape
    Xd = dev(X)
    vals = torch.full((n, k), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((n, k), -1, dtype=torch.int16, device="cuda")
    P.dr_topk(Xd, k, vals, idx)
    torch.cuda.synchronize()
    return vals.cpu().numpy(), host_idx(idx)


# ---------------------------------------------------------------------------------------------------
# (1) D-ReLU
# ---------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("n,D,k", [
    (1003, 64, 16), (1003, 128, 32), (517, 128, 8), (300, 128, 64), (129, 128, 128), (200, 64, 1),
    (257, 8, 3), (131, 33, 7), (99, 100, 25), (64, 256, 32), (33, 1000, 100), (17, 1024, 512), (5, 1, 1),
])
def test_topk_random_rows(n, D, k):
    say(f"topk random n={n} D={D} k={k}")
    rng = np.random.default_rng(100 + D + k)
    X = rng.standard_normal((n, D)).astype(np.float32)
    gv, gi = gpu_topk(X, k)
    ov, oi = oracle.topk(X, k)
    assert np.array_equal(gi, oi)
    assert np.array_equal(gv.astype(np.float64), ov)


@pytest.mark.parametrize("D,k", [(64, 16), (128, 32), (128, 64), (96, 5)])
def test_topk_ties_zeros_and_degenerate_rows(D, k):
    say(f"topk ties D={D} k={k}")
    rng = np.random.default_rng(7)
    n = 400
    X = np.round(rng.standard_normal((n, D)) * 2).astype(np.float32)      # heavy ties
    X[0] = 3.25                                                             # all equal
    X[1] = 0.0
    X[2] = -0.0
    X[3, ::2] = 0.0
    X[3, 1::2] = -0.0                                                       # zeros of both signs
    X[4] = -np.arange(D, dtype=np.float32) - 1                              # all negative, descending
    X[5] = np.arange(D, dtype=np.float32)                                   # ascending: last k columns
    X[6] = np.maximum(X[6], 0)                                              # ReLU-like: many exact zeros
    X[7] = np.float32(1e-40)                                                # denormals
    X[8, :] = np.finfo(np.float32).max
    X[8, 1::3] = -np.finfo(np.float32).max
    gv, gi = gpu_topk(X, k)
    ov, oi = oracle.topk(X, k)
    assert np.array_equal(gi, oi)
    assert np.array_equal(gv.view(np.uint32), ov.astype(np.float32).view(np.uint32))   # bit copies incl. sign of zero


def test_topk_empty_input_is_noop():
    say("topk n=0")
    X = torch.empty((0, 64), dtype=torch.float32, device="cuda")
    P.dr_topk(X, 16, torch.empty((0, 16), device="cuda"), torch.empty((0, 16), dtype=torch.int16, device="cuda"))
    torch.cuda.synchronize()


# ---------------------------------------------------------------------------------------------------
# setup: edge values and stable transpose
# ---------------------------------------------------------------------------------------------------

def _patterns():
    rng = np.random.default_rng(11)
    out = []
    g = make_graph("tiny", seed=0)
    out += [("tiny.near", g.near), ("tiny.pins", g.pins), ("tiny.pinned", g.pinned)]
    rp, ci, _ = random_csr(rng, 700, 300, 12, dup=True)
    out.append(("random.dup", HostPattern(700, 300, rp, ci)))
    rp, ci, _ = random_csr(rng, 1500, 5000, 6, dup=False, evil_rows=(3, 777), evil_deg=3000)
    out.append(("random.evil", HostPattern(1500, 5000, rp, ci)))
    rp, ci, _ = random_csr(rng, 3000, 40, 9, dup=True)       # very long transposed rows
    out.append(("random.tall", HostPattern(3000, 40, rp, ci)))
    rp = np.zeros(11, np.int32)
    out.append(("empty", HostPattern(10, 7, rp, np.zeros(0, np.int32))))
    return out


@pytest.mark.parametrize("name,pat", _patterns(), ids=[n for n, _ in _patterns()])
def test_normalize_and_transpose_bit_exact(name, pat):
    say(f"normalize/transpose {name} M={pat.n_rows} N={pat.n_cols} E={len(pat.colidx)}")
    for mode in (P.DR_NORM_MEAN, P.DR_NORM_SYM):
        A = P.device_relation(pat, mode)
        torch.cuda.synchronize()
        want = oracle.csr_normalize(mode, pat.n_rows, pat.n_cols, pat.rowptr, pat.colidx)
        got = A.vals.cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (name, mode)
    At = P.device_transpose(A)
    o_rp, o_ci, o_v = oracle.csr_transpose(pat.n_rows, pat.n_cols, pat.rowptr, pat.colidx, want)
    assert np.array_equal(At.rowptr.cpu().numpy(), o_rp)
    assert np.array_equal(At.colidx.cpu().numpy(), o_ci)
    assert np.array_equal(At.vals.cpu().numpy().view(np.uint32), o_v.view(np.uint32))
    # pattern-only transpose (no values)
    Ap = P.upload_pattern(pat)
    Atp = P.device_transpose(Ap)
    assert np.array_equal(Atp.colidx.cpu().numpy(), o_ci) and Atp.vals is None


# ---------------------------------------------------------------------------------------------------
# (2) DR-SpMM forward, (3) backward
# ---------------------------------------------------------------------------------------------------

SPMM_CASES = [
    # M, N, max_deg, D, k, dup, evil
    (1000, 900, 12, 64, 16, False, False),
    (1000, 900, 12, 128, 32, True, False),
    (777, 1301, 9, 128, 8, False, True),
    (515, 400, 20, 128, 64, True, True),
    (300, 300, 7, 128, 128, False, False),     # k = D: ordinary SpMM
    (300, 200, 7, 64, 7, True, False),         # odd k: scalar loads
    (300, 200, 7, 96, 6, False, False),        # k % 4 == 2: pair loads
    (200, 150, 5, 1024, 300, False, False),    # wide rows, k above one lane group
    (100, 80, 5, 5, 1, True, False),
    (777, 1301, 9, 128, 2, False, True),       # fewer pairs than lanes in a row group (masked lanes), long rows
    (1000, 900, 12, 128, 4, True, True),
    (600, 500, 10, 64, 12, True, True),        # two strided pairs per lane, the second masked for half the lanes
    (600, 500, 10, 96, 20, False, True),       # three
    (600, 500, 10, 128, 28, True, False),      # four
]


def _spmm_inputs(case, seed):
    M, N, max_deg, D, k, dup, evil = case
    rng = np.random.default_rng(seed)
    ev = (5, M - 1) if evil else ()
    rp, ci, av = random_csr(rng, M, N, max_deg, dup=dup, evil_rows=ev, evil_deg=2500)
    X = rng.standard_normal((N, D)).astype(np.float32)
    return rng, rp, ci, av, X


@pytest.mark.parametrize("case", SPMM_CASES, ids=[f"M{c[0]}_D{c[3]}_k{c[4]}" for c in SPMM_CASES])
def test_spmm_fwd_parity(case):
    M, N, _, D, k, _, _ = case
    say(f"spmm_fwd {case}")
    rng, rp, ci, av, X = _spmm_inputs(case, 21)
    ov, oi = oracle.topk(X, k)
    H_o, l1row, l1elem = oracle.spmm_fwd(rp, ci, av, ov, oi, D, want_l1elem=True)
    A = P.Csr(M, N, dev(rp), dev(ci), dev(av))
    H = torch.full((M, D), float("nan"), dtype=torch.float32, device="cuda")
    P.dr_spmm_fwd(A, dev(ov, torch.float32), dev(oi.astype(np.uint16).view(np.int16)), D, k, H)
    torch.cuda.synchronize()
    H = H.cpu().numpy()
    assert_row_bound(H, H_o, l1row, "spmm_fwd")
    assert_elem_bound(H, H_o, l1elem, "spmm_fwd")


@pytest.mark.parametrize("case", SPMM_CASES, ids=[f"M{c[0]}_D{c[3]}_k{c[4]}" for c in SPMM_CASES])
def test_spmm_bwd_parity(case):
    M, N, _, D, k, _, _ = case
    say(f"spmm_bwd {case}")
    rng, rp, ci, av, X = _spmm_inputs(case, 22)
    _, oi = oracle.topk(X, k)
    dH = rng.standard_normal((M, D)).astype(np.float32)
    t_rp, t_ci, t_v = oracle.csr_transpose(M, N, rp, ci, av)
    G_o, l1row, l1elem = oracle.spmm_bwd(t_rp, t_ci, t_v, dH, oi, want_l1elem=True)
    At = P.Csr(N, M, dev(t_rp), dev(t_ci), dev(t_v))
    idx_d = dev(oi.astype(np.uint16).view(np.int16))
    G = torch.full((N, k), float("nan"), dtype=torch.float32, device="cuda")
    P.dr_spmm_bwd(At, dev(dH), idx_d, D, k, G, accumulate=False)
    torch.cuda.synchronize()
    Gh = G.cpu().numpy()
    assert_row_bound(Gh, G_o, l1row, "spmm_bwd")
    assert_elem_bound(Gh, G_o, l1elem, "spmm_bwd")
    # accumulate: second call adds onto the first result
    P.dr_spmm_bwd(At, dev(dH), idx_d, D, k, G, accumulate=True)
    torch.cuda.synchronize()
    assert_row_bound(G.cpu().numpy(), 2 * G_o, 2 * l1row, "spmm_bwd accumulate")


def test_spmm_on_small_workload_relations():
    """The three relations of the 60k-cell workload, forward and backward, through the device-side
    normalisation and transpose."""
    w = workload("small")
    g = make_graph("small", seed=0)
    T = make_tensors(w["Nc"], w["Nn"], w["D"], seed=0)
    D, k = w["D"], w["k"]
    src = {"near": T.X_cell, "pins": T.X_cell, "pinned": T.X_net}
    for name, pat, mode in (("near", g.near, P.DR_NORM_MEAN), ("pins", g.pins, P.DR_NORM_MEAN),
                            ("pinned", g.pinned, P.DR_NORM_SYM)):
        say(f"small.{name} E={pat.nnz}")
        rel = oracle.relation(pat, mode)
        ov, oi = oracle.topk(src[name], k)
        H_o, l1row, l1elem = oracle.spmm_fwd(rel.rowptr, rel.colidx, rel.vals, ov, oi, D, want_l1elem=True)
        A = P.device_relation(pat, mode)
        n_src = pat.n_cols
        vals = torch.empty((n_src, k), dtype=torch.float32, device="cuda")
        idx = torch.empty((n_src, k), dtype=torch.int16, device="cuda")
        P.dr_topk(dev(src[name]), k, vals, idx)
        H = torch.empty((pat.n_rows, D), dtype=torch.float32, device="cuda")
        P.dr_spmm_fwd(A, vals, idx, D, k, H)
        torch.cuda.synchronize()
        assert np.array_equal(host_idx(idx), oi)
        assert_row_bound(H.cpu().numpy(), H_o, l1row, f"small.{name} fwd")
        assert_elem_bound(H.cpu().numpy(), H_o, l1elem, f"small.{name} fwd")
        dH = np.random.default_rng(5).standard_normal((pat.n_rows, D)).astype(np.float32)
        t = oracle.csr_transpose(pat.n_rows, pat.n_cols, rel.rowptr, rel.colidx, rel.vals)
        G_o, gl1row, gl1elem = oracle.spmm_bwd(*t, dH, oi, want_l1elem=True)
        At = P.device_transpose(A)
        assert np.array_equal(At.colidx.cpu().numpy(), t[1])
        G = torch.empty((n_src, k), dtype=torch.float32, device="cuda")
        P.dr_spmm_bwd(At, dev(dH), idx, D, k, G)
        torch.cuda.synchronize()
        assert_row_bound(G.cpu().numpy(), G_o, gl1row, f"small.{name} bwd")
        assert_elem_bound(G.cpu().numpy(), G_o, gl1elem, f"small.{name} bwd")


# ---------------------------------------------------------------------------------------------------
# the layer
# ---------------------------------------------------------------------------------------------------

def _layer_case(name, seed, **override):
    w = workload(name)
    w.update(override)
    g = make_graph(name, seed=seed, **{k: v for k, v in override.items() if k in ("Nc", "Nn", "grid")})
    T = make_tensors(g.Nc, g.Nn, w["D"], seed=seed)
    return w, g, T


LAYER_CASES = [
    ("tiny", 0, {}),                                               # 2048 cells, D=64, k=16
    ("tiny", 1, dict(Nc=1500, Nn=1000, grid=(50, 30), D=128, k=32)),  # ragged against the 128-row tiles
    ("tiny", 2, dict(Nc=333, Nn=90, grid=(37, 9), D=32, k=5)),
    ("small", 0, {}),                                              # 60 000 cells, 40 000 nets, D=64, k=16
    ("tiny", 3, dict(Nc=700, Nn=450, grid=(35, 20), D=96, k=24)),     # three column slabs, one idle wavefront
    ("tiny", 4, dict(Nc=513, Nn=300, grid=(27, 19), D=64, k=64)),     # k = D: D-ReLU is the identity
]


@pytest.mark.parametrize("name,seed,override", LAYER_CASES, ids=["tiny", "ragged128", "odd32", "small", "D96_k24", "D64_kD"])
def test_heteroconv_fwd_bwd_parity(name, seed, override):
    w, g, T = _layer_case(name, seed, **override)
    D, k = w["D"], w["k"]
    say(f"heteroconv {name} seed={seed} Nc={g.Nc} Nn={g.Nn} D={D} k={k}")
    o_near = oracle.relation(g.near, oracle.NORM_MEAN)
    o_pins = oracle.relation(g.pins, oracle.NORM_MEAN)
    o_pinned = oracle.relation(g.pinned, oracle.NORM_SYM)
    of = oracle.heteroconv_fwd(o_near, o_pins, o_pinned, T.X_cell, T.X_net, T.W, k, k)

    near = P.device_relation(g.near, P.DR_NORM_MEAN)
    pins = P.device_relation(g.pins, P.DR_NORM_MEAN)
    pinned = P.device_relation(g.pinned, P.DR_NORM_SYM)
    layer = P.HeteroConv(near, pins, pinned, D, k, k)
    saved = layer.alloc_saved()
    Wd = {n: dev(T.W[n]) for n in P.WEIGHT_NAMES}
    Y_cell = torch.full((g.Nc, D), float("nan"), dtype=torch.float32, device="cuda")
    Y_net = torch.full((g.Nn, D), float("nan"), dtype=torch.float32, device="cuda")
    layer.heteroconv_fwd(dev(T.X_cell), dev(T.X_net), Wd, Y_cell, Y_net, saved)
    torch.cuda.synchronize()

    # saved CBSR: bit-exact
    assert np.array_equal(host_idx(saved["idx_cell"]), of["idx_cell"])
    assert np.array_equal(host_idx(saved["idx_net"]), of["idx_net"])
    assert np.array_equal(saved["vals_cell"].cpu().numpy().astype(np.float64), of["vals_cell"])
    assert np.array_equal(saved["vals_net"].cpu().numpy().astype(np.float64), of["vals_net"])
    # outputs within the bound
    l1c, l1n = of["l1_cell"], of["l1_net"]
    assert_row_bound(Y_cell.cpu().numpy(), of["Y_cell"], l1c.sum(axis=1), "Y_cell")
    assert_row_bound(Y_net.cpu().numpy(), of["Y_net"], l1n.sum(axis=1), "Y_net")
    assert_elem_bound(Y_cell.cpu().numpy(), of["Y_cell"], l1c, "Y_cell")
    assert_elem_bound(Y_net.cpu().numpy(), of["Y_net"], l1n, "Y_net")
    # the merge mask is a floating-point decision: it must agree wherever the two branches are
    # separated by more than the error bound, and be a valid 0/1 choice elsewhere
    mask = saved["mask"].cpu().numpy()
    assert set(np.unique(mask)) <= {0, 1}
    decided = np.abs(of["Z_near"] - of["Z_pinned"]) > 2e-5 * l1c
    assert decided.mean() > 0.99
    assert np.array_equal(mask[decided], of["mask"][decided])

    # backward on the ORACLE's saved state (identical selections on both sides)
    saved_o = dict(saved)
    saved_o["H_near"] = dev(of["H_near"], torch.float32)
    saved_o["H_pins"] = dev(of["H_pins"], torch.float32)
    saved_o["H_pinned"] = dev(of["H_pinned"], torch.float32)
    saved_o["mask"] = dev(of["mask"])
    ob = oracle.heteroconv_bwd(o_near, o_pins, o_pinned, T.W, of, T.dY_cell, T.dY_net)
    dX_cell = torch.full((g.Nc, D), float("nan"), dtype=torch.float32, device="cuda")
    dX_net = torch.full((g.Nn, D), float("nan"), dtype=torch.float32, device="cuda")
    dW = {n: torch.full((D, D), float("nan"), dtype=torch.float32, device="cuda") for n in P.WEIGHT_NAMES}
    layer.heteroconv_bwd(dev(T.dY_cell), dev(T.dY_net), Wd, saved_o, dX_cell, dX_net, dW)
    torch.cuda.synchronize()
    dXc, dXn = dX_cell.cpu().numpy(), dX_net.cpu().numpy()
    # zero off the saved positions, compact values within the bound
    sel_c = np.zeros((g.Nc, D), bool)
    np.put_along_axis(sel_c, of["idx_cell"].astype(np.int64), True, axis=1)
    sel_n = np.zeros((g.Nn, D), bool)
    np.put_along_axis(sel_n, of["idx_net"].astype(np.int64), True, axis=1)
    assert np.all(dXc[~sel_c] == 0) and np.all(dXn[~sel_n] == 0)
    gc = np.take_along_axis(dXc, of["idx_cell"].astype(np.int64), axis=1)
    gn = np.take_along_axis(dXn, of["idx_net"].astype(np.int64), axis=1)
    # the L1 of the compact gradient counts the terms of the transposed SpMMs and of the self term; the
    # projections feeding them add their own rounding, so allow the row bound only (contract) here
    assert_row_bound(gc, ob["dXs_cell"], ob["l1_dxs_cell"].sum(axis=1), "dX_cell")
    assert_row_bound(gn, ob["dXs_net"], ob["l1_dxs_net"].sum(axis=1), "dX_net")
    # weight gradients: reductions over all rows; bound by the L1 norm of the terms of each entry
    Xs_c = oracle.densify(of["vals_cell"], of["idx_cell"], D)
    Xs_n = oracle.densify(of["vals_net"], of["idx_net"], D)
    dZn = np.where(of["mask"] == 1, T.dY_cell, 0).astype(np.float64)
    dZq = np.where(of["mask"] == 0, T.dY_cell, 0).astype(np.float64)
    l1 = {
        "self_near": np.abs(Xs_c).T @ np.abs(dZn), "neigh_near": np.abs(of["H_near"]).T @ np.abs(dZn),
        "self_pins": np.abs(Xs_n).T @ np.abs(T.dY_net.astype(np.float64)),
        "neigh_pins": np.abs(of["H_pins"]).T @ np.abs(T.dY_net.astype(np.float64)),
        "pinned": np.abs(of["H_pinned"]).T @ np.abs(dZq),
    }
    for n in P.WEIGHT_NAMES:
        assert_row_bound(dW[n].cpu().numpy(), ob["dW"][n], l1[n].sum(axis=1), f"dW.{n}")
        assert_elem_bound(dW[n].cpu().numpy(), ob["dW"][n], l1[n], f"dW.{n}", tol=1e-4)

    # backward on the GPU's own saved state agrees with the oracle wherever the masks agree row-wise
    layer.heteroconv_bwd(dev(T.dY_cell), dev(T.dY_net), Wd, saved, dX_cell, dX_net, dW)
    torch.cuda.synchronize()
    ok = cells_with_agreeing_masks(o_near.rowptr, o_near.colidx, mask, of["mask"])
    assert ok.sum() >= 0.9 * g.Nc, f"only {int(ok.sum())} of {g.Nc} cells have a neighbourhood whose masks agree"
    say(f"   backward on the layer's own saved state: {int(ok.sum())} of {g.Nc} cells compared")
    gc2 = np.take_along_axis(dX_cell.cpu().numpy(), of["idx_cell"].astype(np.int64), axis=1)
    assert_row_bound(gc2[ok], ob["dXs_cell"][ok], ob["l1_dxs_cell"].sum(axis=1)[ok], "dX_cell (own saved)")
    layer.heteroconv_destroy()


def test_heteroconv_transposes_match_oracle():
    g = make_graph("tiny", seed=0)
    say("heteroconv context transposes")
    rels = [P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
            P.device_relation(g.pinned, P.DR_NORM_SYM)]
    layer = P.HeteroConv(*rels, 64, 16, 16)
    import ctypes
    from paper_2508_16769_amd import binding
    for which, (pat, mode) in enumerate(((g.near, 0), (g.pins, 0), (g.pinned, 1))):
        t = layer.heteroconv_get_transpose(which)
        rel = oracle.relation(pat, mode)
        o_rp, o_ci, o_v = oracle.csr_transpose(pat.n_rows, pat.n_cols, rel.rowptr, rel.colidx, rel.vals)
        assert (t.n_rows, t.n_cols, t.nnz) == (pat.n_cols, pat.n_rows, pat.nnz)
        got_ci = torch.empty(pat.nnz, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        binding.hip_runtime().hipMemcpy(
            ctypes.c_void_p(got_ci.data_ptr()), ctypes.c_void_p(t.colidx), ctypes.c_size_t(4 * pat.nnz), 3)
        torch.cuda.synchronize()
        assert np.array_equal(got_ci.cpu().numpy(), o_ci)
    layer.heteroconv_destroy()


def test_heteroconv_is_bit_reproducible_and_stream_agnostic():
    """No atomics on results and fixed summation orders: two runs, with the relations on one stream or on three,
    launched from the default or from a side stream, give bit-identical outputs."""
    w, g, T = _layer_case("tiny", 5, Nc=3000, Nn=2000, grid=(60, 50), D=128, k=32)
    D, k = w["D"], w["k"]
    near = P.device_relation(g.near, P.DR_NORM_MEAN)
    pins = P.device_relation(g.pins, P.DR_NORM_MEAN)
    pinned = P.device_relation(g.pinned, P.DR_NORM_SYM)
    layer = P.HeteroConv(near, pins, pinned, D, k, k)
    Wd = {n: dev(T.W[n]) for n in P.WEIGHT_NAMES}
    Xc, Xn, dYc, dYn = dev(T.X_cell), dev(T.X_net), dev(T.dY_cell), dev(T.dY_net)

    def run(mode, stream):
        layer.heteroconv_set_overlap(mode)
        saved = layer.alloc_saved()
        Yc = torch.full((g.Nc, D), float("nan"), dtype=torch.float32, device="cuda")
        Yn = torch.full((g.Nn, D), float("nan"), dtype=torch.float32, device="cuda")
        dXc, dXn = torch.empty_like(Yc), torch.empty_like(Yn)
        dW = {n: torch.empty((D, D), dtype=torch.float32, device="cuda") for n in P.WEIGHT_NAMES}
        torch.cuda.synchronize()
        layer.heteroconv_fwd(Xc, Xn, Wd, Yc, Yn, saved, stream=stream)
        layer.heteroconv_bwd(dYc, dYn, Wd, saved, dXc, dXn, dW, stream=stream)
        torch.cuda.synchronize()
        return [Yc, Yn, dXc, dXn, saved["mask"], saved["H_near"]] + [dW[n] for n in P.WEIGHT_NAMES]

    side = torch.cuda.Stream()
    ref = run(P.DR_OVERLAP_OFF, None)
    for mode, stream in ((P.DR_OVERLAP_OFF, None), (P.DR_OVERLAP_ON, None), (P.DR_OVERLAP_ON, side), (P.DR_OVERLAP_OFF, side)):
        out = run(mode, stream)
        for a, b in zip(ref, out):
            assert torch.equal(a, b), (mode, stream is side)
    layer.heteroconv_destroy()
