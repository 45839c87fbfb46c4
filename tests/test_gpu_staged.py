"""dr_spmm_bwd_planned (the transposed DR-SpMM with the gathered dH rows staged in LDS tile by tile) against
oracle.spmm_bwd through the C ABI: element and row bounds, exact zeros, independence of the processing order bit
for bit, the accumulate form, widths D = 32 .. 128 and k = 1 .. D, tiles cut by either capacity, refusals."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2508_16769_amd as P
from circuit_synth import make_graph
from gpu_util import assert_elem_bound, assert_row_bound, dev, random_csr, say

pytestmark = pytest.mark.gpu


def _csr(rowptr, colidx, vals, M, N):
    return P.Csr(M, N, dev(rowptr), dev(colidx), dev(vals))


def _run(At, plan, dH, idx, k, accumulate=False, init=None):
    G = torch.full((At.n_rows, k), float("nan"), dtype=torch.float32, device="cuda") if init is None else init.clone()
    plan.dr_spmm_bwd_planned(dH, idx, k, G, accumulate=accumulate)
    torch.cuda.synchronize()
    return G.cpu().numpy()


CASES = [
    # (N rows of At, M columns, max degree, D, k, duplicates)
    (700, 500, 9, 128, 32, False),
    (513, 300, 20, 128, 5, True),
    (300, 4000, 40, 128, 64, False),      # many distinct neighbours: tiles cut by the gathered-row capacity
    (257, 90, 7, 128, 128, True),
    (1000, 800, 12, 64, 16, False),
    (333, 200, 6, 64, 1, True),
    (400, 350, 10, 96, 24, False),
    (129, 60, 5, 32, 32, False),
    (90, 50, 200, 128, 32, True),         # long rows over few neighbours: tiles cut by the edge capacity
    (64, 64, 0, 128, 8, False),           # no edges at all
    (300, 260, 11, 192, 40, False),       # three column slabs
    (210, 180, 9, 256, 64, True),         # four column slabs, four outputs per lane
    (150, 4000, 70, 256, 16, False),      # 256 columns, tiles cut by the gathered-row capacity
]


@pytest.mark.parametrize("N,M,max_deg,D,k,dup", CASES, ids=[f"N{c[0]}_M{c[1]}_deg{c[2]}_D{c[3]}_k{c[4]}" for c in CASES])
def test_planned_bwd_parity_and_order_independence(N, M, max_deg, D, k, dup):
    rng = np.random.default_rng(N + 7 * D + k)
    say(f"dr_spmm_bwd_planned N={N} M={M} max_deg={max_deg} D={D} k={k} dup={dup}")
    rowptr, colidx, vals = random_csr(rng, N, M, max_deg, dup=dup)
    dH = rng.standard_normal((M, D)).astype(np.float32)
    X = rng.standard_normal((N, D)).astype(np.float32)
    _, idx = oracle.topk(X, k)
    want, l1row, l1elem = oracle.spmm_bwd(rowptr, colidx, vals, dH, idx, want_l1elem=True)
    At = _csr(rowptr, colidx, vals, N, M)
    d_dH, d_idx = dev(dH), dev(idx.astype(np.uint16).view(np.int16))
    results = []
    for label, order in (("own order", None), ("reversed", np.arange(N)[::-1].copy()), ("random", rng.permutation(N))):
        plan = P.SpmmPlan(At, D, None if order is None else dev(order.astype(np.int32)))
        n_tiles, reuse = plan.dr_spmm_plan_info()
        got = _run(At, plan, d_dH, d_idx, k)
        assert_row_bound(got, want, l1row, f"G ({label})")
        assert_elem_bound(got, want, l1elem, f"G ({label})")
        results.append(got)
        # accumulate: onto a known start
        start = torch.from_numpy(rng.standard_normal((N, k)).astype(np.float32)).cuda()
        acc = _run(At, plan, d_dH, d_idx, k, accumulate=True, init=start)
        assert np.array_equal(acc, start.cpu().numpy() + got), label
        say(f"   {label}: {n_tiles} tiles, reuse {reuse:.2f}")
        plan.dr_spmm_plan_destroy()
    assert np.array_equal(results[0], results[1]) and np.array_equal(results[0], results[2])
    # the plain kernel sums short rows in the same order: identical bits there
    G = torch.empty((N, k), dtype=torch.float32, device="cuda")
    P.dr_spmm_bwd(At, d_dH, d_idx, D, k, G)
    torch.cuda.synchronize()
    short = np.diff(rowptr) <= 32
    assert np.array_equal(G.cpu().numpy()[short], results[0][short])


def test_planned_bwd_on_a_placed_near_relation():
    """The transposed `near` relation of the small workload in placement order: parity, and the staging reuses rows."""
    g = make_graph("small", seed=0)
    D, k = 64, 16
    rng = np.random.default_rng(5)
    rel = oracle.relation(g.near, oracle.NORM_MEAN)
    t_rp, t_ci, t_v = oracle.csr_transpose(rel.M, rel.N, rel.rowptr, rel.colidx, rel.vals)
    dH = rng.standard_normal((g.Nc, D)).astype(np.float32)
    _, idx = oracle.topk(rng.standard_normal((g.Nc, D)).astype(np.float32), k)
    want, l1row, l1elem = oracle.spmm_bwd(t_rp, t_ci, t_v, dH, idx, want_l1elem=True)
    At = _csr(t_rp, t_ci, t_v, g.Nc, g.Nc)
    plan = P.SpmmPlan(At, D, dev(g.cell_order))
    n_tiles, reuse = plan.dr_spmm_plan_info()
    say(f"small near^T in placement order: {n_tiles} tiles, reuse {reuse:.2f}")
    assert reuse > 3.0
    got = _run(At, plan, dev(dH), dev(idx.astype(np.uint16).view(np.int16)), k)
    assert_row_bound(got, want, l1row, "G")
    assert_elem_bound(got, want, l1elem, "G")
    plain = P.SpmmPlan(At, D, None)
    assert plain.dr_spmm_plan_info()[1] < reuse          # rows of one grid line share fewer neighbours than a square patch


def test_layer_backward_with_a_cell_order_equals_the_layer_without():
    """heteroconv_set_cell_order switches the transposed `near` DR-SpMM of the layer's backward to the staged kernel:
    same gradients (bit for bit on cells that feed at most 32 destinations, where both kernels sum in storage order;
    within the rounding of a different summation order elsewhere), and the whole layer still matches the oracle."""
    from circuit_synth import make_tensors
    g = make_graph("small", seed=0)
    D, k = 64, 16
    T = make_tensors(g.Nc, g.Nn, D, seed=0)
    rels = [P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
            P.device_relation(g.pinned, P.DR_NORM_SYM)]
    layer = P.HeteroConv(*rels, D, k, k)
    saved = layer.alloc_saved()
    Wd = {n: dev(T.W[n]) for n in P.WEIGHT_NAMES}
    Yc = torch.empty((g.Nc, D), device="cuda")
    Yn = torch.empty((g.Nn, D), device="cuda")
    layer.heteroconv_fwd(dev(T.X_cell), dev(T.X_net), Wd, Yc, Yn, saved)

    def backward():
        dXc = torch.full((g.Nc, D), float("nan"), device="cuda")
        dXn = torch.full((g.Nn, D), float("nan"), device="cuda")
        dW = {n: torch.empty((D, D), device="cuda") for n in P.WEIGHT_NAMES}
        layer.heteroconv_bwd(dev(T.dY_cell), dev(T.dY_net), Wd, saved, dXc, dXn, dW)
        torch.cuda.synchronize()
        return dXc.cpu().numpy(), dXn.cpu().numpy(), {n: dW[n].cpu().numpy() for n in dW}

    plain = backward()
    assert layer.heteroconv_set_cell_order(dev(g.cell_order)) is True
    staged = backward()
    out_deg = np.bincount(g.near.colidx, minlength=g.Nc)          # destinations a cell feeds = edges of its row of near^T
    short = out_deg <= 32
    assert short.mean() > 0.9
    assert np.array_equal(plain[0][short], staged[0][short])
    scale = np.abs(plain[0]).sum(axis=1, keepdims=True) + 1e-30
    assert np.all(np.abs(plain[0] - staged[0]) <= 1e-6 * scale)
    assert np.array_equal(plain[1], staged[1])
    for n in P.WEIGHT_NAMES:
        assert np.array_equal(plain[2][n], staged[2][n]), n
    # a random order shares too few neighbours per tile: the layer keeps the plain kernel
    assert layer.heteroconv_set_cell_order(dev(np.random.default_rng(0).permutation(g.Nc).astype(np.int32))) is False
    assert np.array_equal(backward()[0], plain[0])
    layer.heteroconv_destroy()


def test_plan_refusals():
    rng = np.random.default_rng(0)
    lib = P.load()
    # a row with more edges than a tile's record capacity
    rowptr = np.array([0, 3000, 3003], np.int32)
    colidx = rng.integers(0, 50, 3003).astype(np.int32)
    vals = np.ones(3003, np.float32)
    At = _csr(rowptr, colidx, vals, 2, 50)
    with pytest.raises(P.DrError) as e:
        P.SpmmPlan(At, 128)
    assert e.value.code == P.DR_ERR_UNSUPPORTED and "edges" in str(e.value)
    # a row with more distinct neighbours than a tile holds
    rowptr = np.array([0, 600], np.int32)
    At = _csr(rowptr, np.arange(600, dtype=np.int32), np.ones(600, np.float32), 1, 600)
    with pytest.raises(P.DrError) as e:
        P.SpmmPlan(At, 128)
    assert e.value.code == P.DR_ERR_UNSUPPORTED
    # D that the slabs do not divide, an order that is no permutation
    rp, ci, v = random_csr(rng, 50, 40, 5)
    At = _csr(rp, ci, v, 50, 40)
    with pytest.raises(P.DrError) as e:
        P.SpmmPlan(At, 100)
    assert e.value.code == P.DR_ERR_UNSUPPORTED
    with pytest.raises(P.DrError) as e:
        P.SpmmPlan(At, 128, dev(np.zeros(50, np.int32)))
    assert e.value.code == P.DR_ERR_INVALID_ARG and "permutation" in str(e.value)
    plan = P.SpmmPlan(At, 128)
    one = ctypes.c_void_p(256)
    assert lib.dr_spmm_bwd_planned(plan._p, one, one, 129, one, 0, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_spmm_bwd_planned(None, one, one, 8, one, 0, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_spmm_bwd_planned(plan._p, ctypes.c_void_p(260), one, 8, one, 0, None) == P.DR_ERR_INVALID_ARG
