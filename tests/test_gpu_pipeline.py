"""The host-side pipeline (dr_pipeline_*): what a slot holds after submit -> acquire is checked bit for bit against
the oracle's setup functions and against a context built the ordinary way; slots are reused with graphs of other
sizes; protocol errors come back as errors."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_16769_amd as P
from paper_2508_16769_amd.binding import _view
from circuit_synth import make_graph, make_tensors
from gpu_util import dev, say

pytestmark = pytest.mark.gpu

D, K = 64, 16


def _graphs():
    return [make_graph("tiny", seed=30, Nc=3000, Nn=1800, grid=(60, 50)),
            make_graph("tiny", seed=31, Nc=1111, Nn=700, grid=(40, 30)),       # smaller than its slot's first graph
            make_graph("tiny", seed=32, Nc=2500, Nn=2000, grid=(50, 50)),
            make_graph("tiny", seed=33, Nc=3000, Nn=1500, grid=(60, 50))]


def _csr_arrays(c, with_vals=True):
    rp = _view(c.rowptr, (c.n_rows + 1,), torch.int32).cpu().numpy()
    ci = _view(c.colidx, (c.nnz,), torch.int32).cpu().numpy()
    v = _view(c.vals, (c.nnz,), torch.float32).cpu().numpy() if with_vals else None
    return rp, ci, v


def _layer_outputs(layer, Xc, Xn, T, g):
    saved = layer.alloc_saved()
    Wd = {n: dev(T.W[n]) for n in P.WEIGHT_NAMES}
    Yc = torch.empty((g.Nc, D), dtype=torch.float32, device="cuda")
    Yn = torch.empty((g.Nn, D), dtype=torch.float32, device="cuda")
    layer.heteroconv_fwd(Xc, Xn, Wd, Yc, Yn, saved)
    dXc, dXn = torch.empty_like(Yc), torch.empty_like(Yn)
    dW = {n: torch.empty((D, D), dtype=torch.float32, device="cuda") for n in P.WEIGHT_NAMES}
    layer.heteroconv_bwd(dev(T.dY_cell), dev(T.dY_net), Wd, saved, dXc, dXn, dW)
    torch.cuda.synchronize()
    return [Yc, Yn, dXc, dXn] + [dW[n] for n in P.WEIGHT_NAMES]


def test_pipeline_slots_hold_what_the_setup_calls_produce():
    gs = _graphs()
    Ts = [make_tensors(g.Nc, g.Nn, D, seed=40 + i) for i, g in enumerate(gs)]
    pl = P.Pipeline(n_slots=2, n_threads=2, max_cells=3000, max_nets=2000,
                    max_nnz_near=max(g.near.nnz for g in gs), max_nnz_pins=max(g.pins.nnz for g in gs), D=D, k_cell=K, k_net=K)
    say("pipeline: four graphs through two slots")
    order = [(0, 0), (1, 1), (2, 0), (3, 1)]               # (graph, slot): every slot is used twice
    submitted = 0

    def submit(i):
        g, slot = gs[order[i][0]], order[i][1]
        pl.dr_pipeline_submit(slot, g.near.rowptr, g.near.colidx, g.pins.rowptr, g.pins.colidx, Ts[order[i][0]].X_cell,
                              Ts[order[i][0]].X_net)

    submit(0)
    submit(1)
    submitted = 2
    for step, (gi, slot) in enumerate(order):
        g, T = gs[gi], Ts[gi]
        layer, xc, xn = pl.dr_pipeline_acquire(slot)
        torch.cuda.synchronize()
        say(f"pipeline: graph {gi} in slot {slot}: {g.Nc} cells, {g.Nn} nets")
        assert (layer.Nc, layer.Nn) == (g.Nc, g.Nn)
        # ---- relations: patterns as given, pinned = transpose pattern, edge values as the oracle computes them ----
        rel = pl.dr_pipeline_relations(slot)
        o_rel = (oracle.relation(g.near, oracle.NORM_MEAN), oracle.relation(g.pins, oracle.NORM_MEAN),
                 oracle.relation(g.pinned, oracle.NORM_SYM))
        for r, o, name in zip(rel, o_rel, ("near", "pins", "pinned")):
            assert (r.n_rows, r.n_cols, r.nnz) == (o.M, o.N, len(o.colidx)), name
            rp, ci, v = _csr_arrays(r)
            assert np.array_equal(rp, o.rowptr) and np.array_equal(ci, o.colidx), name
            assert np.array_equal(v.view(np.uint32), o.vals.view(np.uint32)), name
        # ---- transposed adjacencies of the slot's context ----
        for which, o in enumerate(o_rel):
            t = layer.heteroconv_get_transpose(which)
            rp, ci, v = _csr_arrays(t)
            o_rp, o_ci, o_v = oracle.csr_transpose(o.M, o.N, o.rowptr, o.colidx, o.vals)
            assert np.array_equal(rp, o_rp) and np.array_equal(ci, o_ci) and np.array_equal(v.view(np.uint32), o_v.view(np.uint32))
        # ---- uploaded embeddings ----
        assert np.array_equal(_view(xc, (g.Nc, D), torch.float32).cpu().numpy(), T.X_cell)
        assert np.array_equal(_view(xn, (g.Nn, D), torch.float32).cpu().numpy(), T.X_net)
        # ---- the layer on the slot's context = the layer on a context built the ordinary way, bit for bit ----
        got = _layer_outputs(layer, xc, xn, T, g)
        ref_layer = P.HeteroConv(P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
                                 P.device_relation(g.pinned, P.DR_NORM_SYM), D, K, K)
        want = _layer_outputs(ref_layer, dev(T.X_cell), dev(T.X_net), T, g)
        for a, b in zip(got, want):
            assert torch.equal(a, b)
        ref_layer.heteroconv_destroy()
        pl.dr_pipeline_release(slot)
        if submitted < len(order):                          # refill the slot that has just been released
            submit(submitted)
            submitted += 1
    pl.dr_pipeline_destroy()


def test_pipeline_protocol_errors():
    g = make_graph("tiny", seed=5, Nc=500, Nn=300, grid=(25, 20))
    say("pipeline: protocol errors")
    pl = P.Pipeline(n_slots=1, n_threads=1, max_cells=500, max_nets=300, max_nnz_near=g.near.nnz, max_nnz_pins=g.pins.nnz,
                    D=D, k_cell=K, k_net=K)
    with pytest.raises(P.DrError):
        pl.dr_pipeline_acquire(0)                           # nothing submitted
    with pytest.raises(P.DrError):
        pl.dr_pipeline_release(0)
    big = make_graph("tiny", seed=6, Nc=600, Nn=300, grid=(30, 20))
    with pytest.raises(P.DrError) as e:
        pl.dr_pipeline_submit(0, big.near.rowptr, big.near.colidx, big.pins.rowptr, big.pins.colidx)
    assert "capacity" in str(e.value)
    pl.dr_pipeline_submit(0, g.near.rowptr, g.near.colidx, g.pins.rowptr, g.pins.colidx)
    with pytest.raises(P.DrError):
        pl.dr_pipeline_submit(0, g.near.rowptr, g.near.colidx, g.pins.rowptr, g.pins.colidx)   # slot busy
    with pytest.raises(P.DrError):
        pl.dr_pipeline_submit(1, g.near.rowptr, g.near.colidx, g.pins.rowptr, g.pins.colidx)   # no such slot
    layer, xc, xn = pl.dr_pipeline_acquire(0)
    assert xc is None and xn is None                        # no embeddings were given
    with pytest.raises(P.DrError):
        pl.dr_pipeline_acquire(0)                           # already acquired
    pl.dr_pipeline_release(0)
    pl.dr_pipeline_destroy()
    with pytest.raises(P.DrError):
        P.Pipeline(n_slots=0, n_threads=1, max_cells=10, max_nets=10, max_nnz_near=10, max_nnz_pins=10, D=D, k_cell=K, k_net=K)


def test_training_steps_on_pipeline_slots_equal_steps_on_ordinary_contexts():
    """One model over the contexts of two pipeline slots trains on a stream of sub-graph pairs (the slots are re-bound
    between steps, to graphs of other sizes); every step equals, bit for bit, the step of a model built the ordinary
    way for that pair."""
    L, D2, k = 2, 64, 16
    pairs = [(make_graph("tiny", seed=70, Nc=2000, Nn=1300, grid=(50, 40)), make_graph("tiny", seed=71, Nc=1800, Nn=1400, grid=(50, 40))),
             (make_graph("tiny", seed=72, Nc=1500, Nn=900, grid=(50, 30)), make_graph("tiny", seed=73, Nc=2000, Nn=1400, grid=(50, 40)))]
    gs = [g for p in pairs for g in p]
    rng = np.random.default_rng(8)
    feats = {id(g): (rng.standard_normal((g.Nc, D2)).astype(np.float32), rng.standard_normal((g.Nn, D2)).astype(np.float32),
                     rng.standard_normal(g.Nc).astype(np.float32)) for g in gs}
    n_par = P.hgnn_num_params(L, D2)
    theta0 = rng.uniform(-0.2, 0.2, n_par).astype(np.float32)
    say("pipeline: training steps on re-bound slot contexts")
    pl = P.Pipeline(2, 2, 2000, 1400, max(g.near.nnz for g in gs), max(g.pins.nnz for g in gs), D2, k, k)

    def state():
        return (dev(theta0), torch.zeros(n_par, dtype=torch.float32, device="cuda"), torch.zeros(n_par, dtype=torch.float32, device="cuda"),
                torch.full((n_par,), float("nan"), dtype=torch.float32, device="cuda"), torch.full((1,), float("nan"), dtype=torch.float32, device="cuda"))

    th, m, v, gr, ls = state()
    model = None
    for step, pair in enumerate(pairs, start=1):
        for slot, g in enumerate(pair):
            pl.dr_pipeline_submit(slot, g.near.rowptr, g.near.colidx, g.pins.rowptr, g.pins.colidx, feats[id(g)][0], feats[id(g)][1])
        got = [pl.dr_pipeline_acquire(slot) for slot in range(2)]
        if model is None:
            model = P.Hgnn([a[0] for a in got], L)          # the slot contexts; their addresses do not change
        tg = [dev(feats[id(g)][2]) for g in pair]
        model.hgnn_train_step([a[1] for a in got], [a[2] for a in got], tg, th, m, v, 2e-4, 0.9, 0.999, 1e-8, 1e-5, step, gr, ls)
        torch.cuda.synchronize()
        for slot in range(2):
            pl.dr_pipeline_release(slot)
        # the same step on ordinary contexts, from the same parameter state
        keep = [(P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN), P.device_relation(g.pinned, P.DR_NORM_SYM))
                for g in pair]
        ctxs = [P.HeteroConv(d[0], d[1], d[2], D2, k, k) for d in keep]
        ref = P.Hgnn(ctxs, L)
        if step == 1:
            th_r, m_r, v_r, gr_r, ls_r = state()
        ref.hgnn_train_step([dev(feats[id(g)][0]) for g in pair], [dev(feats[id(g)][1]) for g in pair], tg, th_r, m_r, v_r,
                            2e-4, 0.9, 0.999, 1e-8, 1e-5, step, gr_r, ls_r)
        torch.cuda.synchronize()
        assert torch.equal(ls, ls_r) and torch.equal(gr, gr_r) and torch.equal(th, th_r), step
        assert np.isfinite(float(ls.cpu()[0]))
        ref.hgnn_destroy()
        for c in ctxs:
            c.heteroconv_destroy()
    model.hgnn_destroy()
    pl.dr_pipeline_destroy()


def test_pipeline_with_an_edgeless_relation():
    """A sub-graph whose near relation has no edges at all (and nets that pin nothing for a few rows): the slot still
    delivers a usable context and the layer equals the ordinary one bit for bit."""
    from circuit_synth.generate import Pattern, transpose_pattern
    g = make_graph("tiny", seed=90, Nc=600, Nn=400, grid=(30, 20))
    near = Pattern(g.Nc, g.Nc, np.zeros(g.Nc + 1, dtype=np.int32), np.zeros(0, dtype=np.int32))
    say("pipeline: edgeless near relation")
    T = make_tensors(g.Nc, g.Nn, D, seed=91)
    pl = P.Pipeline(1, 1, g.Nc, g.Nn, 16, g.pins.nnz, D, K, K)
    pl.dr_pipeline_submit(0, near.rowptr, near.colidx, g.pins.rowptr, g.pins.colidx, T.X_cell, T.X_net)
    layer, xc, xn = pl.dr_pipeline_acquire(0)

    class G2:
        Nc, Nn = g.Nc, g.Nn
    got = _layer_outputs(layer, xc, xn, T, G2)
    ref = P.HeteroConv(P.device_relation(near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
                       P.device_relation(transpose_pattern(g.pins), P.DR_NORM_SYM), D, K, K)
    want = _layer_outputs(ref, dev(T.X_cell), dev(T.X_net), T, G2)
    for a, b in zip(got, want):
        assert torch.equal(a, b)
    assert torch.isfinite(got[0]).all()
    ref.heteroconv_destroy()
    pl.dr_pipeline_release(0)
    pl.dr_pipeline_destroy()
