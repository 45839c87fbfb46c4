"""Parity of the multi-layer training step (hgnn_train_step) with the oracle, through the C ABI.

A later layer's discrete decisions (top-k, max-merge, ReLU sign) depend on fp32 values the earlier layers
produced, so every layer is compared "teacher-forced": the oracle recomputes that layer from the very inputs /
saved selections the HIP path used (read back through hgnn_get_layer_buffers).  Selections must then match bit
for bit and values within the row bound; the read-out, the loss, the gradient sums and the Adam update are checked
the same way, and the loss of the whole step is compared with the free-running oracle as an end-to-end sanity."""
import numpy as np
import pytest
import torch

import oracle
from oracle import hgnn as ohgnn
import paper_2508_16769_amd as P
from circuit_synth import make_graph
from gpu_util import assert_row_bound, dev, host_idx, say

pytestmark = pytest.mark.gpu

LR, B1, B2, EPS, WD = 2e-4, 0.9, 0.999, 1e-8, 1e-5


def _setup(n_graphs, Nc, Nn, grid, D, k, L, seed0=20):
    rng = np.random.default_rng(seed0)
    graphs, rels, ctxs, keep = [], [], [], []
    Xc, Xn, tg = [], [], []
    for q in range(n_graphs):
        g = make_graph("small", seed=seed0 + q, Nc=Nc + 64 * q, Nn=Nn + 32 * q, grid=grid)
        graphs.append(g)
        rels.append((oracle.relation(g.near, oracle.NORM_MEAN), oracle.relation(g.pins, oracle.NORM_MEAN),
                     oracle.relation(g.pinned, oracle.NORM_SYM)))
        d = (P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
             P.device_relation(g.pinned, P.DR_NORM_SYM))
        keep.append(d)
        ctxs.append(P.HeteroConv(d[0], d[1], d[2], D, k, k))
        Xc.append(rng.standard_normal((g.Nc, D)).astype(np.float32))
        Xn.append(rng.standard_normal((g.Nn, D)).astype(np.float32))
        tg.append(rng.standard_normal(g.Nc).astype(np.float32))
    bound = np.sqrt(6.0 / (2 * D))
    theta = rng.uniform(-bound, bound, P.hgnn_num_params(L, D)).astype(np.float32)
    return graphs, rels, ctxs, keep, Xc, Xn, tg, theta


def _wgrad_bounds(saved, Xs_c, Xs_n, dYc, dYn, mask):
    """Element-wise sum of |terms| for each of the five weight gradients (dW = A^T B)."""
    dZn, dZq = np.abs(dYc) * (mask == 1), np.abs(dYc) * (mask == 0)
    return dict(self_near=np.abs(Xs_c).T @ dZn, neigh_near=np.abs(saved["H_near"]).T @ dZn,
                self_pins=np.abs(Xs_n).T @ np.abs(dYn), neigh_pins=np.abs(saved["H_pins"]).T @ np.abs(dYn),
                pinned=np.abs(saved["H_pinned"]).T @ dZq)


def _check_layer(model, rels, Ws, q, l, L, D, k, X0=None, check_dw=True):
    """Teacher-forced comparison of sub-graph q, layer l; returns the buffers (numpy) of that layer."""
    b = {kk: (vv.cpu().numpy() if torch.is_tensor(vv) else {n: t.cpu().numpy() for n, t in vv.items()})
         for kk, vv in model.hgnn_get_layer_buffers(q, l).items() if vv is not None}
    if l == 0 and X0 is not None:
        assert np.array_equal(b["X_cell"], X0[0]) and np.array_equal(b["X_net"], X0[1])
    # ---- forward of this layer from the inputs the HIP path used ----
    of = oracle.heteroconv_fwd(*rels[q], b["X_cell"], b["X_net"], Ws[l], k, k)
    assert np.array_equal(host_idx(torch.from_numpy(b["idx_cell"])), of["idx_cell"]), (q, l)
    assert np.array_equal(host_idx(torch.from_numpy(b["idx_net"])), of["idx_net"]), (q, l)
    assert np.array_equal(b["vals_cell"].astype(np.float64), of["vals_cell"])
    want_c, want_n = of["Y_cell"], of["Y_net"]
    if l < L - 1:
        want_c, want_n = np.maximum(want_c, 0), np.maximum(want_n, 0)
        assert (b["Y_cell"] >= 0).all() and (b["Y_net"] >= 0).all()
    assert_row_bound(b["Y_cell"], want_c, of["l1_cell"].sum(axis=1), f"g{q} l{l} Y_cell")
    assert_row_bound(b["Y_net"], want_n, of["l1_net"].sum(axis=1), f"g{q} l{l} Y_net")
    decided = np.abs(of["Z_near"] - of["Z_pinned"]) > 2e-5 * of["l1_cell"]
    assert decided.mean() > 0.98
    assert np.array_equal(b["mask"][decided], of["mask"][decided])
    # ---- backward of this layer from the state and the gradient the HIP path used ----
    saved = {n: b[n] for n in ("vals_cell", "vals_net", "H_near", "H_pins", "H_pinned", "mask")}
    saved["idx_cell"] = host_idx(torch.from_numpy(b["idx_cell"]))
    saved["idx_net"] = host_idx(torch.from_numpy(b["idx_net"]))
    ob = oracle.heteroconv_bwd(*rels[q], Ws[l], saved, b["dY_cell"], b["dY_net"])
    ic, inn = saved["idx_cell"].astype(np.int64), saved["idx_net"].astype(np.int64)
    want_gc, want_gn = ob["dXs_cell"].copy(), ob["dXs_net"].copy()
    if l >= 1:       # the ReLU in front of the layer gates its input gradient
        want_gc *= np.take_along_axis(b["X_cell"], ic, axis=1) > 0
        want_gn *= np.take_along_axis(b["X_net"], inn, axis=1) > 0
    assert_row_bound(np.take_along_axis(b["dX_cell"], ic, axis=1), want_gc, ob["l1_dxs_cell"].sum(axis=1), f"g{q} l{l} dX_cell")
    assert_row_bound(np.take_along_axis(b["dX_net"], inn, axis=1), want_gn, ob["l1_dxs_net"].sum(axis=1), f"g{q} l{l} dX_net")
    off = np.ones(b["dX_cell"].shape, bool)
    np.put_along_axis(off, ic, False, axis=1)
    assert np.all(b["dX_cell"][off] == 0)
    Xs_c = oracle.densify(saved["vals_cell"], saved["idx_cell"], D)
    Xs_n = oracle.densify(saved["vals_net"], saved["idx_net"], D)
    bounds = _wgrad_bounds({n: np.asarray(saved[n], np.float64) for n in ("H_near", "H_pins", "H_pinned")}, Xs_c, Xs_n,
                           b["dY_cell"].astype(np.float64), b["dY_net"].astype(np.float64), saved["mask"])
    for i, n in enumerate(P.WEIGHT_NAMES):
        err = np.abs(b["dW"][n].astype(np.float64) - ob["dW"][n])
        assert not check_dw or np.all(err <= 1e-5 * bounds[n] + 1e-30), (q, l, n, err.max())
    return b


@pytest.mark.parametrize("case", [dict(n_graphs=3, Nc=2400, Nn=1700, grid=(64, 42), D=128, k=32, L=3),
                                  dict(n_graphs=2, Nc=1500, Nn=900, grid=(52, 32), D=64, k=16, L=2)],
                         ids=["3x2400_D128_k32_L3", "2x1500_D64_k16_L2"])
def test_train_step_parity(case):
    n_graphs, D, k, L = case["n_graphs"], case["D"], case["k"], case["L"]
    graphs, rels, ctxs, keep, Xc, Xn, tg, theta0 = _setup(**case)
    say(f"hgnn: {n_graphs} sub-graphs, D={D}, k={k}, L={L}")
    model = P.Hgnn(ctxs, L)
    model.hgnn_set_inspection(True)              # the first layer's dX is checked too
    n_par = P.hgnn_num_params(L, D)
    theta = dev(theta0)
    m = torch.zeros(n_par, dtype=torch.float32, device="cuda")
    v = torch.zeros(n_par, dtype=torch.float32, device="cuda")
    grad = torch.full((n_par,), float("nan"), dtype=torch.float32, device="cuda")
    loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    dXc, dXn, dtg = [dev(a) for a in Xc], [dev(a) for a in Xn], [dev(a) for a in tg]
    model.hgnn_train_step(dXc, dXn, dtg, theta, m, v, LR, B1, B2, EPS, WD, 1, grad, loss)
    torch.cuda.synchronize()

    Ws, w_head = ohgnn.unpack(theta0.astype(np.float64), L, D)
    n_total = sum(g.Nc for g in graphs)
    sq_sum = 0.0
    g_layers = np.zeros(n_par - D)
    g_head = np.zeros(D)
    for q in range(n_graphs):
        last = None
        for l in range(L):
            b = _check_layer(model, rels, Ws, q, l, L, D, k, X0=(Xc[q], Xn[q]))
            for i, n in enumerate(P.WEIGHT_NAMES):
                lo = (l * 5 + i) * D * D
                g_layers[lo:lo + D * D] += b["dW"][n].astype(np.float64).ravel()
            last = b
        # ---- read-out, residual, gradient of the last layer's output ----
        Y = last["Y_cell"].astype(np.float64)
        pred = Y @ w_head
        l1 = np.abs(Y) @ np.abs(w_head)
        assert np.all(np.abs(last["pred"] - pred) <= 1e-5 * l1 + 1e-30)
        r = last["pred"].astype(np.float64) - tg[q]
        sq_sum += float(np.sum(r * r))
        assert np.allclose(last["dpred"], 2.0 * r / n_total, rtol=2e-6, atol=0)
        want_dY = np.outer(last["dpred"].astype(np.float64), w_head)
        assert np.allclose(last["dY_cell"], want_dY, rtol=2e-6, atol=1e-30)
        assert np.all(last["dY_net"] == 0)
        g_head += Y.T @ last["dpred"].astype(np.float64)
    # ---- loss, gradient sums, Adam ----
    loss_gpu = float(loss.cpu()[0])
    assert abs(loss_gpu - sq_sum / n_total) <= 1e-5 * (sq_sum / n_total)
    gg = grad.cpu().numpy().astype(np.float64)
    assert np.allclose(gg[:n_par - D], g_layers, rtol=1e-5, atol=1e-9)
    assert np.allclose(gg[n_par - D:], g_head, rtol=1e-4, atol=1e-7)
    th2, m2, v2 = ohgnn.adam_step(theta0.astype(np.float64), gg, np.zeros(n_par), np.zeros(n_par), LR, B1, B2, EPS, WD, 1)
    assert np.allclose(theta.cpu().numpy(), th2, rtol=0, atol=2e-7 * max(1.0, np.abs(th2).max()) + LR * 1e-3)
    assert np.allclose(m.cpu().numpy(), m2, rtol=1e-5, atol=1e-12)
    assert np.allclose(v.cpu().numpy(), v2, rtol=1e-5, atol=1e-20)
    # ---- the free-running oracle agrees on the loss (discrete flips, if any, are rare and local) ----
    free = ohgnn.train_step(rels, Xc, Xn, tg, theta0.astype(np.float64), np.zeros(n_par), np.zeros(n_par), L, D, k,
                            LR, B1, B2, EPS, WD, 1)
    assert abs(loss_gpu - free["loss"]) <= 1e-3 * free["loss"], (loss_gpu, free["loss"])
    cos = float(gg @ free["grad"] / (np.linalg.norm(gg) * np.linalg.norm(free["grad"])))
    assert cos > 0.999, cos
    # the default model skips what training does not need (first layer's input gradient, last layer's net output and
    # whatever only feeds those): same loss, gradient and update
    fast = P.Hgnn(ctxs, L)
    th_f, m_f, v_f = dev(theta0), torch.zeros_like(m), torch.zeros_like(v)
    gr_f, ls_f = torch.full_like(grad, float("nan")), torch.full_like(loss, float("nan"))
    fast.hgnn_train_step(dXc, dXn, dtg, th_f, m_f, v_f, LR, B1, B2, EPS, WD, 1, gr_f, ls_f)
    torch.cuda.synchronize()
    assert torch.equal(gr_f, grad) and torch.equal(ls_f, loss) and torch.equal(th_f, theta)
    first, last = fast.hgnn_get_layer_buffers(0, 0), fast.hgnn_get_layer_buffers(0, L - 1)
    assert first["dX_cell"] is None and last["Y_net"] is None and last["H_pins"] is None and last["Y_cell"] is not None
    fast.hgnn_destroy()
    # a second step runs from the updated state and lowers nothing it should not touch
    model.hgnn_train_step(dXc, dXn, dtg, theta, m, v, LR, B1, B2, EPS, WD, 2, grad, loss)
    torch.cuda.synchronize()
    assert np.isfinite(float(loss.cpu()[0])) and np.isfinite(theta.cpu().numpy()).all()
    model.hgnn_destroy()
    for c in ctxs:
        c.heteroconv_destroy()


def _check_layer_ks(model, rels, Ws, q, l, L, D, ks, X0=None):
    """Teacher-forced comparison of one layer of a sub-graph that has one K per edge type (dense dX)."""
    from oracle import per_relation as opr
    b = {kk: (vv.cpu().numpy() if torch.is_tensor(vv) else {n: t.cpu().numpy() for n, t in vv.items()})
         for kk, vv in model.hgnn_get_layer_buffers(q, l).items() if vv is not None}
    if l == 0 and X0 is not None:
        assert np.array_equal(b["X_cell"], X0[0]) and np.array_equal(b["X_net"], X0[1])
    of = opr.heteroconv_fwd(*rels[q], b["X_cell"], b["X_net"], Ws[l], ks)
    mine = {"cell_near": "cell", "net_pinned": "net",
            "cell_pins": "cell_pins" if ks.pins != ks.near else "cell", "net_self": "net_self" if ks.self_ != ks.pinned else "net"}
    saved = {n: b[n] for n in ("H_near", "H_pins", "H_pinned", "mask")}
    for theirs, m in mine.items():
        idx = host_idx(torch.from_numpy(b["idx_" + m]))
        assert np.array_equal(idx, of["idx_" + theirs]), (q, l, theirs)
        assert np.array_equal(b["vals_" + m].astype(np.float64), of["vals_" + theirs]), (q, l, theirs)
        saved["idx_" + theirs], saved["vals_" + theirs] = idx, b["vals_" + m]
    want_c, want_n = of["Y_cell"], of["Y_net"]
    if l < L - 1:
        want_c, want_n = np.maximum(want_c, 0), np.maximum(want_n, 0)
    assert_row_bound(b["Y_cell"], want_c, of["l1_cell"].sum(axis=1), f"g{q} l{l} Y_cell")
    assert_row_bound(b["Y_net"], want_n, of["l1_net"].sum(axis=1), f"g{q} l{l} Y_net")
    decided = np.abs(of["Z_near"] - of["Z_pinned"]) > 2e-5 * of["l1_cell"]
    assert np.array_equal(b["mask"][decided], of["mask"][decided])
    ob = opr.heteroconv_bwd(*rels[q], Ws[l], saved, b["dY_cell"], b["dY_net"])
    want_gc, want_gn = ob["dX_cell"].copy(), ob["dX_net"].copy()
    if l >= 1:
        want_gc *= b["X_cell"] > 0
        want_gn *= b["X_net"] > 0
    assert_row_bound(b["dX_cell"], want_gc, ob["l1_dX_cell"].sum(axis=1), f"g{q} l{l} dX_cell")
    assert_row_bound(b["dX_net"], want_gn, ob["l1_dX_net"].sum(axis=1), f"g{q} l{l} dX_net")
    assert np.all(b["dX_cell"][ob["l1_dX_cell"] == 0] == 0) and np.all(b["dX_net"][ob["l1_dX_net"] == 0] == 0)
    Xs_c = oracle.densify(saved["vals_cell_near"], saved["idx_cell_near"], D)
    Xs_n = oracle.densify(saved["vals_net_self"], saved["idx_net_self"], D)
    bounds = _wgrad_bounds({n: np.asarray(saved[n], np.float64) for n in ("H_near", "H_pins", "H_pinned")}, Xs_c, Xs_n,
                           b["dY_cell"].astype(np.float64), b["dY_net"].astype(np.float64), saved["mask"])
    for n in P.WEIGHT_NAMES:
        err = np.abs(b["dW"][n].astype(np.float64) - ob["dW"][n])
        assert np.all(err <= 1e-5 * bounds[n] + 1e-30), (q, l, n, err.max())
    return b


def test_train_step_with_own_k_per_subgraph():
    """Three sub-graphs that share the parameters and keep their own K: one K per edge type (all different), one K
    per edge type with the cells sharing a selection, and one K per node type.  Every layer is checked teacher-forced;
    the loss and the batch gradient are checked against the sums of what the layers produced and the free oracle."""
    from oracle.per_relation import Ks
    D, L = 128, 2
    graphs, rels, ctxs, keep, Xc, Xn, tg, theta0 = _setup(3, 2000, 1400, (64, 42), D, 8, L, seed0=60)
    for c in ctxs:
        c.heteroconv_destroy()
    kset = [Ks.per_relation(8, 32, 16), Ks.per_relation(16, 16, 4), 24]
    ctxs = [P.HeteroConv(*keep[0], D, per_relation=(8, 32, 16)), P.HeteroConv(*keep[1], D, per_relation=(16, 16, 4)),
            P.HeteroConv(*keep[2], D, 24, 24)]
    say("hgnn: three sub-graphs with their own K")
    model = P.Hgnn(ctxs, L)
    model.hgnn_set_inspection(True)
    n_par = P.hgnn_num_params(L, D)
    theta = dev(theta0)
    m = torch.zeros(n_par, dtype=torch.float32, device="cuda")
    v = torch.zeros(n_par, dtype=torch.float32, device="cuda")
    grad = torch.full((n_par,), float("nan"), dtype=torch.float32, device="cuda")
    loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    dXc, dXn, dtg = [dev(a) for a in Xc], [dev(a) for a in Xn], [dev(a) for a in tg]   # kept alive: layer 0 reads them back
    model.hgnn_train_step(dXc, dXn, dtg, theta, m, v, LR, B1, B2, EPS, WD, 1, grad, loss)
    torch.cuda.synchronize()
    Ws, w_head = ohgnn.unpack(theta0.astype(np.float64), L, D)
    n_total = sum(g.Nc for g in graphs)
    sq_sum, g_layers, g_head = 0.0, np.zeros(n_par - D), np.zeros(D)
    for q in range(3):
        for l in range(L):
            if isinstance(kset[q], Ks):
                b = _check_layer_ks(model, rels, Ws, q, l, L, D, kset[q], X0=(Xc[q], Xn[q]))
            else:
                b = _check_layer(model, rels, Ws, q, l, L, D, kset[q], X0=(Xc[q], Xn[q]))
            for i, n in enumerate(P.WEIGHT_NAMES):
                lo = (l * 5 + i) * D * D
                g_layers[lo:lo + D * D] += b["dW"][n].astype(np.float64).ravel()
        r = b["pred"].astype(np.float64) - tg[q]
        sq_sum += float(np.sum(r * r))
        g_head += b["Y_cell"].astype(np.float64).T @ b["dpred"].astype(np.float64)
    loss_gpu = float(loss.cpu()[0])
    assert abs(loss_gpu - sq_sum / n_total) <= 1e-5 * (sq_sum / n_total)
    gg = grad.cpu().numpy().astype(np.float64)
    assert np.allclose(gg[:n_par - D], g_layers, rtol=1e-5, atol=1e-9)
    assert np.allclose(gg[n_par - D:], g_head, rtol=1e-4, atol=1e-7)
    free = ohgnn.train_step(rels, Xc, Xn, tg, theta0.astype(np.float64), np.zeros(n_par), np.zeros(n_par), L, D, kset,
                            LR, B1, B2, EPS, WD, 1)
    assert abs(loss_gpu - free["loss"]) <= 1e-3 * free["loss"], (loss_gpu, free["loss"])
    cos = float(gg @ free["grad"] / (np.linalg.norm(gg) * np.linalg.norm(free["grad"])))
    assert cos > 0.999, cos
    model.hgnn_destroy()
    for c in ctxs:
        c.heteroconv_destroy()


def test_full_size_step_of_eight_subgraphs():
    """The batch of the training-step configuration: 8 independent sub-graphs of 20 000 cells / 14 000 nets,
    3 layers, D = 128, k = 32.  Two (sub-graph, layer) pairs are recomputed by the oracle; the loss, the gradient
    sums and the update are checked for the whole batch."""
    from circuit_synth import workload
    import time
    w = workload("subgraph")
    D, k, L, n_graphs = w["D"], w["k"], 3, 8
    rng = np.random.default_rng(77)
    graphs, rels, ctxs, keep, dXc, dXn, dtg, tgs = [], {}, [], [], [], [], [], []
    for q in range(n_graphs):
        g = make_graph("subgraph", seed=q)
        graphs.append(g)
        d = (P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
             P.device_relation(g.pinned, P.DR_NORM_SYM))
        keep.append(d)
        ctxs.append(P.HeteroConv(d[0], d[1], d[2], D, k, k))
        dXc.append(dev(rng.standard_normal((g.Nc, D)).astype(np.float32)))
        dXn.append(dev(rng.standard_normal((g.Nn, D)).astype(np.float32)))
        tgs.append(rng.standard_normal(g.Nc).astype(np.float32))
        dtg.append(dev(tgs[-1]))
    say(f"hgnn full size: {n_graphs} x ({graphs[0].Nc} cells, {graphs[0].Nn} nets), D={D}, k={k}, L={L}")
    model = P.Hgnn(ctxs, L)
    model.hgnn_set_inspection(True)                   # the oracle checks below read every buffer of a layer
    n_par = P.hgnn_num_params(L, D)
    bound = np.sqrt(6.0 / (2 * D))
    theta0 = rng.uniform(-bound, bound, n_par).astype(np.float32)
    theta = dev(theta0)
    m = torch.zeros(n_par, dtype=torch.float32, device="cuda")
    v = torch.zeros(n_par, dtype=torch.float32, device="cuda")
    grad = torch.empty(n_par, dtype=torch.float32, device="cuda")
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    model.hgnn_train_step(dXc, dXn, dtg, theta, m, v, LR, B1, B2, EPS, WD, 1, grad, loss)
    torch.cuda.synchronize()
    Ws, w_head = ohgnn.unpack(theta0.astype(np.float64), L, D)
    for q, l in ((5, 2), (2, 1)):
        g = graphs[q]
        rels[q] = (oracle.relation(g.near, oracle.NORM_MEAN), oracle.relation(g.pins, oracle.NORM_MEAN),
                   oracle.relation(g.pinned, oracle.NORM_SYM))
        say(f"hgnn full size: oracle on sub-graph {q}, layer {l}")
        _check_layer(model, rels, Ws, q, l, L, D, k)
    n_total = sum(g.Nc for g in graphs)
    sq, g_layers, g_head = 0.0, np.zeros(n_par - D), np.zeros(D)
    for q in range(n_graphs):
        for l in range(L):
            b = model.hgnn_get_layer_buffers(q, l)
            for i, n in enumerate(P.WEIGHT_NAMES):
                lo = (l * 5 + i) * D * D
                g_layers[lo:lo + D * D] += b["dW"][n].cpu().numpy().astype(np.float64).ravel()
        Y = b["Y_cell"].cpu().numpy().astype(np.float64)
        pred = b["pred"].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(pred - Y @ w_head) <= 1e-5 * (np.abs(Y) @ np.abs(w_head)))
        r = pred - tgs[q]
        sq += float(np.sum(r * r))
        g_head += Y.T @ b["dpred"].cpu().numpy().astype(np.float64)
    assert abs(float(loss.cpu()[0]) - sq / n_total) <= 1e-5 * sq / n_total
    gg = grad.cpu().numpy().astype(np.float64)
    assert np.allclose(gg[:n_par - D], g_layers, rtol=1e-5, atol=1e-9)
    assert np.allclose(gg[n_par - D:], g_head, rtol=1e-4, atol=1e-7)
    th2, m2, v2 = ohgnn.adam_step(theta0.astype(np.float64), gg, np.zeros(n_par), np.zeros(n_par), LR, B1, B2, EPS, WD, 1)
    assert np.allclose(theta.cpu().numpy(), th2, rtol=0, atol=2e-7 + LR * 1e-3)
    # timing of the step (reported, not asserted), without the parts only inspection needs
    model.hgnn_set_inspection(False)
    for _ in range(2):
        model.hgnn_train_step(dXc, dXn, dtg, theta, m, v, LR, B1, B2, EPS, WD, 2, grad, loss)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(10):
        model.hgnn_train_step(dXc, dXn, dtg, theta, m, v, LR, B1, B2, EPS, WD, 3 + i, grad, loss)
    torch.cuda.synchronize()
    say(f"hgnn full size: {(time.perf_counter() - t0) * 100:.3f} ms per training step, loss {float(loss.cpu()[0]):.5f}")
    model.hgnn_destroy()
    # the same batch stacked into one graph by the library: same first step, one launch per kernel
    batched = P.Hgnn(ctxs, L, batched=True)
    th_b = dev(theta0)
    m_b, v_b = torch.zeros_like(m), torch.zeros_like(v)
    grad_b, loss_b = torch.empty_like(grad), torch.empty_like(loss)
    batched.hgnn_train_step(dXc, dXn, dtg, th_b, m_b, v_b, LR, B1, B2, EPS, WD, 1, grad_b, loss_b)
    torch.cuda.synchronize()
    assert abs(float(loss_b.cpu()[0]) - sq / n_total) <= 1e-5 * sq / n_total
    assert np.allclose(grad_b.cpu().numpy(), gg, rtol=1e-4, atol=1e-6 * np.abs(gg).max())
    for _ in range(2):
        batched.hgnn_train_step(dXc, dXn, dtg, th_b, m_b, v_b, LR, B1, B2, EPS, WD, 2, grad_b, loss_b)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(10):
        batched.hgnn_train_step(dXc, dXn, dtg, th_b, m_b, v_b, LR, B1, B2, EPS, WD, 3 + i, grad_b, loss_b)
    torch.cuda.synchronize()
    say(f"hgnn full size, batched: {(time.perf_counter() - t0) * 100:.3f} ms per training step (inputs gathered each step)")
    batched.hgnn_destroy()
    for c in ctxs:
        c.heteroconv_destroy()


@pytest.mark.skip(reason="Capturing hgnn_train_step into a HIP graph ended in a host segmentation fault inside the call "
                         "(record: all sub-graphs had been enqueued with status 0; the fault came after that, on the capturing "
                         "thread, in the part of the step that joins the sub-graph streams back into the caller's stream).  "
                         "What the code did at that point and a capture does not allow for: the sub-graphs' launches were "
                         "appended to the one capture from several host threads at once (the enqueue workers), on streams that "
                         "entered the capture only through an event wait issued from those other threads.  The cause has not "
                         "been shown on the host side, so the capture is not run on the GPU; the library has no capture path.")
def test_graph_replay_matches_eager_steps():
    """Three training steps replayed from one captured HIP graph equal three eager steps bit for bit (every replay is
    compared, with eager work and synchronisations between the replays)."""
    D, k, L = 128, 32, 2
    graphs, rels, ctxs, keep, Xc, Xn, tg, theta0 = _setup(4, 1200, 800, (40, 30), D, k, L)
    Xc, Xn, tg = [dev(a) for a in Xc], [dev(a) for a in Xn], [dev(a) for a in tg]
    n_par = P.hgnn_num_params(L, D)

    def state():
        return (dev(theta0), torch.zeros(n_par, device="cuda"), torch.zeros(n_par, device="cuda"),
                torch.empty(n_par, device="cuda"), torch.empty(1, device="cuda"))

    model = P.Hgnn(ctxs, L)
    th_e, m_e, v_e, g_e, l_e = state()
    eager = []
    for step in (1, 1, 1):      # the captured step carries step = 1; each eager reference restarts from the same state
        th_e, m_e, v_e, g_e, l_e = state()
        model.hgnn_train_step(Xc, Xn, tg, th_e, m_e, v_e, LR, B1, B2, EPS, WD, step, g_e, l_e)
        torch.cuda.synchronize()
        eager.append((th_e.clone(), g_e.clone(), l_e.clone()))
    th, m, v, g, l = state()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        model.hgnn_train_step(Xc, Xn, tg, th, m, v, LR, B1, B2, EPS, WD, 1, g, l)
    for want in eager:
        th.copy_(dev(theta0)); m.zero_(); v.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(th, want[0]) and torch.equal(g, want[1]) and torch.equal(l, want[2])
    model.hgnn_destroy()


def test_block_diagonal_batch_equals_separate_subgraphs():
    """Independent sub-graphs stacked into one block-diagonal graph give the same step (one launch per kernel
    for the whole batch instead of one per sub-graph): same selections, same loss and gradient up to the order
    of the fp32 sums over rows."""
    from circuit_synth import block_diagonal
    D, k, L, n_graphs = 64, 16, 2, 3
    rng = np.random.default_rng(5)
    gs = [make_graph("small", seed=40 + q, Nc=1800 + 100 * q, Nn=1100 + 50 * q, grid=(50, 40)) for q in range(n_graphs)]
    Xc = [rng.standard_normal((g.Nc, D)).astype(np.float32) for g in gs]
    Xn = [rng.standard_normal((g.Nn, D)).astype(np.float32) for g in gs]
    tg = [rng.standard_normal(g.Nc).astype(np.float32) for g in gs]
    n_par = P.hgnn_num_params(L, D)
    theta0 = rng.uniform(-0.2, 0.2, n_par).astype(np.float32)

    def step(graph_list, xc, xn, t):
        keep, ctxs = [], []
        for g in graph_list:
            d = (P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
                 P.device_relation(g.pinned, P.DR_NORM_SYM))
            keep.append(d)
            ctxs.append(P.HeteroConv(d[0], d[1], d[2], D, k, k))
        model = P.Hgnn(ctxs, L)
        th = dev(theta0)
        m = torch.zeros(n_par, dtype=torch.float32, device="cuda")
        v = torch.zeros(n_par, dtype=torch.float32, device="cuda")
        gr = torch.empty(n_par, dtype=torch.float32, device="cuda")
        ls = torch.empty(1, dtype=torch.float32, device="cuda")
        model.hgnn_train_step([dev(a) for a in xc], [dev(a) for a in xn], [dev(a) for a in t], th, m, v, LR, B1, B2, EPS, WD, 1, gr, ls)
        torch.cuda.synchronize()
        idx = [host_idx(model.hgnn_get_layer_buffers(q, L - 1)["idx_cell"]) for q in range(len(graph_list))]
        out = float(ls.cpu()[0]), gr.cpu().numpy().astype(np.float64), np.concatenate(idx)
        model.hgnn_destroy()
        for c in ctxs:
            c.heteroconv_destroy()
        return out

    loss_a, grad_a, idx_a = step(gs, Xc, Xn, tg)
    big = block_diagonal(gs)
    assert big.Nc == sum(g.Nc for g in gs) and big.near.nnz == sum(g.near.nnz for g in gs)
    loss_b, grad_b, idx_b = step([big], [np.concatenate(Xc)], [np.concatenate(Xn)], [np.concatenate(tg)])
    assert np.array_equal(idx_a, idx_b)                      # last layer's selections: bit-identical inputs reached it
    assert abs(loss_a - loss_b) <= 1e-6 * abs(loss_a)
    assert np.allclose(grad_a, grad_b, rtol=1e-4, atol=1e-6 * np.abs(grad_a).max())


@pytest.mark.parametrize("contiguous", [False, True], ids=["scattered_inputs", "contiguous_inputs"])
def test_batched_model_stacks_the_subgraphs_on_the_device(contiguous):
    """hgnn_create_batched: the library stacks the batch into one block-diagonal graph itself.  Its step is checked
    (a) bit for bit against a one-graph model built from the host-side block-diagonal graph, (b) layer by layer
    against the oracle through the per-sub-graph views of the stacked buffers, (c) against the streamed model."""
    from circuit_synth import block_diagonal
    D, k, L, n_graphs = 128, 32, 2, 3
    rng = np.random.default_rng(6)
    gs = [make_graph("small", seed=50 + q, Nc=1700 + 130 * q, Nn=1000 + 70 * q, grid=(50, 40)) for q in range(n_graphs)]
    say(f"hgnn batched: {n_graphs} sub-graphs, contiguous inputs: {contiguous}")
    Xc = [rng.standard_normal((g.Nc, D)).astype(np.float32) for g in gs]
    Xn = [rng.standard_normal((g.Nn, D)).astype(np.float32) for g in gs]
    tg = [rng.standard_normal(g.Nc).astype(np.float32) for g in gs]
    n_par = P.hgnn_num_params(L, D)
    bound = np.sqrt(6.0 / (2 * D))
    theta0 = rng.uniform(-bound, bound, n_par).astype(np.float32)

    def contexts(graph_list):
        keep = [(P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
                 P.device_relation(g.pinned, P.DR_NORM_SYM)) for g in graph_list]
        return keep, [P.HeteroConv(d[0], d[1], d[2], D, k, k) for d in keep]

    def tensors():
        if not contiguous:
            return [dev(a) for a in Xc], [dev(a) for a in Xn], [dev(a) for a in tg], None
        allc, alln, allt = dev(np.concatenate(Xc)), dev(np.concatenate(Xn)), dev(np.concatenate(tg))
        oc = np.cumsum([0] + [g.Nc for g in gs])
        on = np.cumsum([0] + [g.Nn for g in gs])
        return ([allc[oc[q]:oc[q + 1]] for q in range(n_graphs)], [alln[on[q]:on[q + 1]] for q in range(n_graphs)],
                [allt[oc[q]:oc[q + 1]] for q in range(n_graphs)], (allc, alln, allt))

    def run(model, xs):
        th = dev(theta0)
        m = torch.zeros(n_par, dtype=torch.float32, device="cuda")
        v = torch.zeros(n_par, dtype=torch.float32, device="cuda")
        gr = torch.full((n_par,), float("nan"), dtype=torch.float32, device="cuda")
        ls = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
        model.hgnn_train_step(xs[0], xs[1], xs[2], th, m, v, LR, B1, B2, EPS, WD, 1, gr, ls)
        torch.cuda.synchronize()
        return float(ls.cpu()[0]), gr.cpu().numpy(), th.cpu().numpy()

    keep, ctxs = contexts(gs)
    xs = tensors()
    batched = P.Hgnn(ctxs, L, batched=True)
    batched.hgnn_set_inspection(True)
    loss_b, grad_b, theta_b = run(batched, xs)
    # (a) the host-side block-diagonal graph as one sub-graph: identical launches, identical bits
    keep1, ctx1 = contexts([block_diagonal(gs)])
    one = P.Hgnn(ctx1, L)
    x1 = ([dev(np.concatenate(Xc))], [dev(np.concatenate(Xn))], [dev(np.concatenate(tg))])
    loss_1, grad_1, theta_1 = run(one, x1)
    assert loss_b == loss_1 and np.array_equal(grad_b, grad_1) and np.array_equal(theta_b, theta_1)
    # (b) per-sub-graph views of the stacked buffers against the oracle, teacher-forced
    rels = [(oracle.relation(g.near, oracle.NORM_MEAN), oracle.relation(g.pins, oracle.NORM_MEAN),
             oracle.relation(g.pinned, oracle.NORM_SYM)) for g in gs]
    Ws, w_head = ohgnn.unpack(theta0.astype(np.float64), L, D)
    for q, l in ((0, 0), (1, 1), (2, 0), (2, 1)):
        b = _check_layer(batched, rels, Ws, q, l, L, D, k, X0=(Xc[q], Xn[q]), check_dw=False)
    r = b["pred"].astype(np.float64) - tg[2]
    assert np.allclose(b["dpred"], 2.0 * r / sum(g.Nc for g in gs), rtol=2e-6, atol=0)
    # (c) the streamed model of the same contexts: same step up to the order of the sums over rows
    streamed = P.Hgnn(ctxs, L)
    loss_s, grad_s, theta_s = run(streamed, xs)
    assert abs(loss_b - loss_s) <= 1e-6 * abs(loss_s)
    assert np.allclose(grad_b, grad_s, rtol=1e-4, atol=1e-6 * np.abs(grad_s).max())
    # contexts with different K cannot share one launch
    other = P.HeteroConv(*keep[0], D, 16, 16)
    with pytest.raises(P.DrError):
        P.Hgnn([ctxs[0], other], L, batched=True)
    for mdl in (batched, one, streamed):
        mdl.hgnn_destroy()
    for c in ctxs + ctx1 + [other]:
        c.heteroconv_destroy()


def test_rejects_bad_arguments():
    g = make_graph("tiny", seed=0)
    d = (P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
         P.device_relation(g.pinned, P.DR_NORM_SYM))
    ctx = P.HeteroConv(d[0], d[1], d[2], 64, 16, 16)
    with pytest.raises(P.DrError):
        P.Hgnn([ctx, ctx], 2)                 # one context cannot serve two sub-graphs of a batch
    with pytest.raises(P.DrError):
        P.Hgnn([ctx], 0)
    model = P.Hgnn([ctx], 1)
    n = P.hgnn_num_params(1, 64)
    z = torch.zeros(n, dtype=torch.float32, device="cuda")
    x = [torch.zeros((g.Nc, 64), device="cuda")], [torch.zeros((g.Nn, 64), device="cuda")], [torch.zeros(g.Nc, device="cuda")]
    with pytest.raises(P.DrError):
        model.hgnn_train_step(x[0], x[1], x[2], z, z.clone(), z.clone(), LR, B1, B2, EPS, WD, 0, z.clone(), z[:1].clone())
    model.hgnn_destroy()
    ctx.heteroconv_destroy()


def test_batched_model_with_one_k_per_edge_type():
    """Stacking also serves contexts that keep one K per edge type (the same triple for the whole batch): same step
    as the streamed model up to the order of the fp32 sums over rows, same selections."""
    D, L, kk = 96, 2, (8, 24, 12)
    rng = np.random.default_rng(9)
    gs = [make_graph("small", seed=80 + q, Nc=1300 + 90 * q, Nn=800 + 40 * q, grid=(40, 40)) for q in range(3)]
    say("hgnn batched with k_near/k_pins/k_pinned = %s" % (kk,))
    Xc = [dev(rng.standard_normal((g.Nc, D)).astype(np.float32)) for g in gs]
    Xn = [dev(rng.standard_normal((g.Nn, D)).astype(np.float32)) for g in gs]
    tg = [dev(rng.standard_normal(g.Nc).astype(np.float32)) for g in gs]
    n_par = P.hgnn_num_params(L, D)
    theta0 = rng.uniform(-0.15, 0.15, n_par).astype(np.float32)
    keep = [(P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
             P.device_relation(g.pinned, P.DR_NORM_SYM)) for g in gs]
    ctxs = [P.HeteroConv(*d, D, per_relation=kk) for d in keep]
    out = []
    for batched in (False, True):
        model = P.Hgnn(ctxs, L, batched=batched)
        th = dev(theta0)
        m = torch.zeros(n_par, dtype=torch.float32, device="cuda")
        v = torch.zeros(n_par, dtype=torch.float32, device="cuda")
        gr = torch.empty(n_par, dtype=torch.float32, device="cuda")
        ls = torch.empty(1, dtype=torch.float32, device="cuda")
        model.hgnn_train_step(Xc, Xn, tg, th, m, v, LR, B1, B2, EPS, WD, 1, gr, ls)
        torch.cuda.synchronize()
        b = model.hgnn_get_layer_buffers(1, 0)
        out.append((float(ls.cpu()[0]), gr.cpu().numpy().astype(np.float64), host_idx(b["idx_cell"]), host_idx(b["idx_cell_pins"]),
                    host_idx(b["idx_net_self"]), b["Y_cell"].cpu().numpy()))
        model.hgnn_destroy()
    (la, ga, i1a, i2a, i3a, ya), (lb, gb, i1b, i2b, i3b, yb) = out
    assert np.array_equal(i1a, i1b) and np.array_equal(i2a, i2b) and np.array_equal(i3a, i3b)
    assert i1a.shape[1] == kk[0] and i2a.shape[1] == kk[1] and i3a.shape[1] == kk[1]
    assert np.array_equal(ya, yb)                     # first layer: same inputs, same kernels, same rows
    assert abs(la - lb) <= 1e-6 * abs(la)
    assert np.allclose(ga, gb, rtol=1e-4, atol=1e-6 * np.abs(ga).max())
    for c in ctxs:
        c.heteroconv_destroy()
