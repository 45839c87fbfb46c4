"""HeteroConv with one K per edge type (heteroconv_create_per_relation) against the fp64 oracle
(oracle/per_relation.py), element by element, on graphs that span several tiles with ragged tails."""
import numpy as np
import pytest
import torch

import oracle
from oracle import per_relation as opr
import paper_2508_16769_amd as P
from circuit_synth import make_graph, make_tensors
from gpu_util import assert_elem_bound, assert_row_bound, dev, host_idx, say

pytestmark = pytest.mark.gpu

# (seed, Nc, Nn, grid, D, (k_near, k_pins, k_pinned))
CASES = [
    (0, 1500, 1000, (50, 30), 128, (8, 32, 16)),     # three different widths, k_near < k_pins
    (1, 1500, 1000, (50, 30), 128, (32, 4, 64)),     # k_near > k_pins, wide pinned
    (2, 777, 500, (37, 21), 64, (16, 16, 4)),        # cells share one selection, nets do not
    (3, 777, 500, (37, 21), 64, (2, 8, 8)),          # nets share one selection, cells do not
    (4, 700, 450, (35, 20), 96, (24, 96, 1)),        # three column slabs; k = D and k = 1
    (5, 333, 90, (37, 9), 32, (5, 3, 32)),
    (6, 1500, 1000, (50, 30), 128, (70, 66, 68)),    # more pairs per row than the register-resident part holds
    (7, 20000, 14000, (200, 100), 128, (4, 16, 8)),  # a training sub-graph
]


def _ids():
    return [f"Nc{c[1]}_D{c[4]}_k{'-'.join(map(str, c[5]))}" for c in CASES]


def _support(idx, D):
    sel = np.zeros((idx.shape[0], D), bool)
    np.put_along_axis(sel, idx.astype(np.int64), True, axis=1)
    return sel


@pytest.mark.parametrize("case", CASES, ids=_ids())
def test_per_relation_fwd_bwd_parity(case):
    seed, Nc, Nn, grid, D, kk = case
    say(f"per-relation heteroconv seed={seed} Nc={Nc} Nn={Nn} D={D} k_near/k_pins/k_pinned={kk}")
    g = make_graph("tiny", seed=seed, Nc=Nc, Nn=Nn, grid=grid)
    T = make_tensors(g.Nc, g.Nn, D, seed=seed)
    ks = opr.Ks.per_relation(*kk)
    rel = (oracle.relation(g.near, oracle.NORM_MEAN), oracle.relation(g.pins, oracle.NORM_MEAN),
           oracle.relation(g.pinned, oracle.NORM_SYM))
    of = opr.heteroconv_fwd(*rel, T.X_cell, T.X_net, T.W, ks)

    near = P.device_relation(g.near, P.DR_NORM_MEAN)
    pins = P.device_relation(g.pins, P.DR_NORM_MEAN)
    pinned = P.device_relation(g.pinned, P.DR_NORM_SYM)
    layer = P.HeteroConv(near, pins, pinned, D, per_relation=kk)
    assert layer.heteroconv_get_k() == (kk[0], kk[1], kk[1], kk[2])
    saved = layer.alloc_saved()
    Wd = {n: dev(T.W[n]) for n in P.WEIGHT_NAMES}
    Y_cell = torch.full((g.Nc, D), float("nan"), dtype=torch.float32, device="cuda")
    Y_net = torch.full((g.Nn, D), float("nan"), dtype=torch.float32, device="cuda")
    layer.heteroconv_fwd(dev(T.X_cell), dev(T.X_net), Wd, Y_cell, Y_net, saved)
    torch.cuda.synchronize()

    # every selection the layer saved: bit-exact
    names = {"cell": "cell_near", "net": "net_pinned", "cell_pins": "cell_pins", "net_self": "net_self"}
    for mine, theirs in names.items():
        if "idx_" + mine not in saved:
            continue
        assert np.array_equal(host_idx(saved["idx_" + mine]), of["idx_" + theirs]), mine
        assert np.array_equal(saved["vals_" + mine].cpu().numpy().astype(np.float64), of["vals_" + theirs]), mine
    assert ("idx_cell_pins" in saved) == (kk[1] != kk[0]) and ("idx_net_self" in saved) == (kk[1] != kk[2])

    for n in ("H_near", "H_pins", "H_pinned"):
        got = saved[n].cpu().numpy()
        assert np.all(np.isfinite(got)), n
    l1c, l1n = of["l1_cell"], of["l1_net"]
    assert_row_bound(Y_cell.cpu().numpy(), of["Y_cell"], l1c.sum(axis=1), "Y_cell")
    assert_row_bound(Y_net.cpu().numpy(), of["Y_net"], l1n.sum(axis=1), "Y_net")
    assert_elem_bound(Y_cell.cpu().numpy(), of["Y_cell"], l1c, "Y_cell")
    assert_elem_bound(Y_net.cpu().numpy(), of["Y_net"], l1n, "Y_net")
    mask = saved["mask"].cpu().numpy()
    assert set(np.unique(mask)) <= {0, 1}
    decided = np.abs(of["Z_near"] - of["Z_pinned"]) > 2e-5 * l1c
    assert np.array_equal(mask[decided], of["mask"][decided])

    # backward on the oracle's saved state (identical selections and mask on both sides)
    saved_o = dict(saved)
    for n in ("H_near", "H_pins", "H_pinned"):
        saved_o[n] = dev(of[n], torch.float32)
    saved_o["mask"] = dev(of["mask"])
    ob = opr.heteroconv_bwd(*rel, T.W, of, T.dY_cell, T.dY_net)
    dX_cell = torch.full((g.Nc, D), float("nan"), dtype=torch.float32, device="cuda")
    dX_net = torch.full((g.Nn, D), float("nan"), dtype=torch.float32, device="cuda")
    dW = {n: torch.full((D, D), float("nan"), dtype=torch.float32, device="cuda") for n in P.WEIGHT_NAMES}
    layer.heteroconv_bwd(dev(T.dY_cell), dev(T.dY_net), Wd, saved_o, dX_cell, dX_net, dW)
    torch.cuda.synchronize()
    dXc, dXn = dX_cell.cpu().numpy(), dX_net.cpu().numpy()
    # exactly zero outside the union of the two selections of a node type; within the bound inside
    sup_c = _support(of["idx_cell_near"], D) | _support(of["idx_cell_pins"], D)
    sup_n = _support(of["idx_net_self"], D) | _support(of["idx_net_pinned"], D)
    assert np.all(dXc[~sup_c] == 0) and np.all(dXn[~sup_n] == 0)
    assert_row_bound(dXc, ob["dX_cell"], ob["l1_dX_cell"].sum(axis=1), "dX_cell")
    assert_row_bound(dXn, ob["dX_net"], ob["l1_dX_net"].sum(axis=1), "dX_net")
    # per element: the projections that feed the gathered terms add their own rounding, so the element bound
    # is the contract's 1e-4 on the element's own terms plus a share of the row's
    err_c = np.abs(dXc - ob["dX_cell"])
    assert np.all(err_c <= 1e-4 * ob["l1_dX_cell"] + 1e-6 * ob["l1_dX_cell"].sum(axis=1, keepdims=True))
    err_n = np.abs(dXn - ob["dX_net"])
    assert np.all(err_n <= 1e-4 * ob["l1_dX_net"] + 1e-6 * ob["l1_dX_net"].sum(axis=1, keepdims=True))

    Xs_c = oracle.densify(of["vals_cell_near"], of["idx_cell_near"], D)
    Xs_n = oracle.densify(of["vals_net_self"], of["idx_net_self"], D)
    dZn = np.where(of["mask"] == 1, T.dY_cell, 0).astype(np.float64)
    dZq = np.where(of["mask"] == 0, T.dY_cell, 0).astype(np.float64)
    dYn = np.abs(T.dY_net.astype(np.float64))
    l1 = {
        "self_near": np.abs(Xs_c).T @ np.abs(dZn), "neigh_near": np.abs(of["H_near"]).T @ np.abs(dZn),
        "self_pins": np.abs(Xs_n).T @ dYn, "neigh_pins": np.abs(of["H_pins"]).T @ dYn,
        "pinned": np.abs(of["H_pinned"]).T @ np.abs(dZq),
    }
    for n in P.WEIGHT_NAMES:
        assert_row_bound(dW[n].cpu().numpy(), ob["dW"][n], l1[n].sum(axis=1), f"dW.{n}")
        assert_elem_bound(dW[n].cpu().numpy(), ob["dW"][n], l1[n], f"dW.{n}", tol=1e-4)

    # one stream or three: same bits
    layer.heteroconv_set_overlap(P.DR_OVERLAP_OFF)
    dX2 = torch.empty_like(dX_cell)
    dXn2 = torch.empty_like(dX_net)
    layer.heteroconv_bwd(dev(T.dY_cell), dev(T.dY_net), Wd, saved_o, dX2, dXn2, dW)
    torch.cuda.synchronize()
    assert torch.equal(dX2, dX_cell) and torch.equal(dXn2, dX_net)
    layer.heteroconv_destroy()


def test_per_relation_with_equal_k_is_the_per_node_type_layer_bit_for_bit():
    g = make_graph("tiny", seed=9, Nc=1500, Nn=1000, grid=(50, 30))
    D, k = 128, 32
    T = make_tensors(g.Nc, g.Nn, D, seed=9)
    say("per-relation with equal k vs heteroconv_create")
    rels = [P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
            P.device_relation(g.pinned, P.DR_NORM_SYM)]
    Wd = {n: dev(T.W[n]) for n in P.WEIGHT_NAMES}
    outs = []
    for layer in (P.HeteroConv(*rels, D, k, k), P.HeteroConv(*rels, D, per_relation=(k, k, k))):
        saved = layer.alloc_saved()
        assert "idx_cell_pins" not in saved and "idx_net_self" not in saved
        Yc = torch.empty((g.Nc, D), dtype=torch.float32, device="cuda")
        Yn = torch.empty((g.Nn, D), dtype=torch.float32, device="cuda")
        layer.heteroconv_fwd(dev(T.X_cell), dev(T.X_net), Wd, Yc, Yn, saved)
        dXc, dXn = torch.empty_like(Yc), torch.empty_like(Yn)
        dW = {n: torch.empty((D, D), dtype=torch.float32, device="cuda") for n in P.WEIGHT_NAMES}
        layer.heteroconv_bwd(dev(T.dY_cell), dev(T.dY_net), Wd, saved, dXc, dXn, dW)
        torch.cuda.synchronize()
        outs.append((Yc, Yn, dXc, dXn, dW))
        layer.heteroconv_destroy()
    for a, b in zip(outs[0][:4], outs[1][:4]):
        assert torch.equal(a, b)
    for n in P.WEIGHT_NAMES:
        assert torch.equal(outs[0][4][n], outs[1][4][n])


def test_per_relation_argument_errors():
    g = make_graph("tiny", seed=0)
    rels = [P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
            P.device_relation(g.pinned, P.DR_NORM_SYM)]
    say("per-relation argument errors")
    for kk in ((0, 4, 4), (4, 65, 4), (4, 4, -1)):
        with pytest.raises(P.DrError) as e:
            P.HeteroConv(*rels, 64, per_relation=kk)
        assert e.value.code == P.DR_ERR_INVALID_ARG
    layer = P.HeteroConv(*rels, 64, per_relation=(4, 8, 16))
    saved = layer.alloc_saved()
    del saved["idx_cell_pins"]                          # a required buffer left out
    X = torch.zeros((g.Nc, 64), device="cuda")
    Xn = torch.zeros((g.Nn, 64), device="cuda")
    Wd = {n: torch.zeros((64, 64), device="cuda") for n in P.WEIGHT_NAMES}
    with pytest.raises(P.DrError) as e:
        layer.heteroconv_fwd(X, Xn, Wd, torch.empty_like(X), torch.empty_like(Xn), saved)
    assert e.value.code == P.DR_ERR_INVALID_ARG and "vals_cell_pins" in str(e.value)
    layer.heteroconv_destroy()


def test_profile_k_times_every_candidate_and_picks_the_fastest():
    """Optimal-K profiling of a training-size sub-graph: a positive time for every (relation, K), best_k is the
    arg-min of the returned table, and a context built from it runs."""
    g = make_graph("subgraph", seed=3)
    D = 128
    T = make_tensors(g.Nc, g.Nn, D, seed=3)
    rels = [P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
            P.device_relation(g.pinned, P.DR_NORM_SYM)]
    say(f"profile_k: sub-graph of {g.Nc} cells / {g.Nn} nets")
    ctx = P.HeteroConv(*rels, D, 1, 1)
    cand = (2, 4, 8, 16, 32, 64)
    Xc, Xn = dev(T.X_cell), dev(T.X_net)
    ms_f, ms_b, best = ctx.heteroconv_profile_k(Xc, Xn, cand, warmup=2, reps=5)
    for r, name in enumerate(("near", "pins", "pinned")):
        say(f"  {name:7s} fwd ms " + " ".join(f"{v:.4f}" for v in ms_f[r]) + " | bwd ms " + " ".join(f"{v:.4f}" for v in ms_b[r]))
        tot = np.array(ms_f[r]) + np.array(ms_b[r])
        assert np.all(np.array(ms_f[r]) > 0) and np.all(np.array(ms_b[r]) > 0)
        assert best[r] == cand[int(np.argmin(tot))]
        # more kept values never make the kernels markedly faster
        assert tot[-1] > 0.8 * tot[0]
    say(f"  best k_near/k_pins/k_pinned = {best}")
    # the embeddings were only read
    assert np.array_equal(Xc.cpu().numpy(), T.X_cell) and np.array_equal(Xn.cpu().numpy(), T.X_net)
    tuned = P.HeteroConv(*rels, D, per_relation=best)
    saved = tuned.alloc_saved()
    Wd = {n: dev(T.W[n]) for n in P.WEIGHT_NAMES}
    Yc = torch.empty((g.Nc, D), dtype=torch.float32, device="cuda")
    Yn = torch.empty((g.Nn, D), dtype=torch.float32, device="cuda")
    tuned.heteroconv_fwd(Xc, Xn, Wd, Yc, Yn, saved)
    torch.cuda.synchronize()
    assert torch.isfinite(Yc).all() and torch.isfinite(Yn).all()
    # argument errors come back before anything is launched
    for bad in ((), (0, 4), (4, 129)):
        with pytest.raises(P.DrError) as e:
            ctx.heteroconv_profile_k(Xc, Xn, bad)
        assert e.value.code == P.DR_ERR_INVALID_ARG
    with pytest.raises(P.DrError):
        ctx.heteroconv_profile_k(Xc, Xn, cand, reps=0)
    tuned.heteroconv_destroy()
    ctx.heteroconv_destroy()
