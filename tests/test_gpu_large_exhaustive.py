"""Every element of the three spec steps at the benchmark's full size (1.2 M cells, 0.9 M nets, D = 128,
k = 32), through the C ABI in the launch configuration bench.py times: dr_topk of all 2.1 M rows bit-exact with
oracle.topk; dr_spmm_fwd and dr_spmm_bwd of the three whole relations against oracle.spmm_fwd / oracle.spmm_bwd, with
the row bound 1e-4 x (L1 norm of the row's terms), the element bound 1e-5 x (L1 norm of the element's terms) and
exact zeros where no term contributes.  The upstream gradients of the backward are the workload's seeded N(0,1)
tensors of the destination type."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
import paper_2508_16769_amd as P
import sampled_checks as sc
from gpu_util import assert_elem_bound, assert_row_bound, dev, host_idx, say

pytestmark = pytest.mark.gpu

K = 32
RELATIONS = (("near", "cell", "cell"), ("pins", "cell", "net"), ("pinned", "net", "cell"))   # name, source type, destination type


@pytest.fixture(scope="module")
def inputs():
    return sc.make_inputs("large")


@pytest.fixture(scope="module")
def whole(inputs):
    return sc.oracle_whole(inputs, K)


@pytest.fixture(scope="module")
def cbsr(inputs):
    """dr_topk of both node types on the device."""
    out = {}
    for key in ("cell", "net"):
        X = inputs["dT"][f"X_{key}"]
        vals = torch.full((X.shape[0], K), float("nan"), dtype=torch.float32, device="cuda")
        idx = torch.full((X.shape[0], K), -1, dtype=torch.int16, device="cuda")
        say(f"large: dr_topk.{key} on {X.shape[0]} rows")
        P.dr_topk(X, K, vals, idx)
        out[key] = (vals, idx)
    torch.cuda.synchronize()
    return out


def test_topk_every_row_is_bit_exact(inputs, whole, cbsr):
    for key in ("cell", "net"):
        vals, idx = cbsr[key]
        assert np.array_equal(host_idx(idx), whole[f"idx_{key}"]), key
        assert np.array_equal(vals.cpu().numpy().astype(np.float64), whole[f"vals_{key}"]), key


@pytest.mark.parametrize("name,src,dst", RELATIONS, ids=[r[0] for r in RELATIONS])
def test_spmm_fwd_every_element(inputs, whole, cbsr, name, src, dst):
    D = inputs["D"]
    A = inputs["dev_rel"][name]
    vals, idx = cbsr[src]
    H = torch.full((A.n_rows, D), float("nan"), dtype=torch.float32, device="cuda")
    say(f"large: dr_spmm_fwd.{name}, {A.nnz} edges")
    P.dr_spmm_fwd(A, vals, idx, D, K, H)
    torch.cuda.synchronize()
    want, l1row, l1elem = whole[f"H_{name}"]
    got = H.cpu().numpy()
    worst = assert_row_bound(got, want, l1row, f"H_{name}")
    assert_elem_bound(got, want, l1elem, f"H_{name}")
    say(f"   {got.shape[0]} rows x {D}: worst err / row L1 = {worst:.2e}")


def test_spmm_bwd_every_element(inputs, whole):
    D, T, tr = inputs["D"], inputs["T"], inputs["tr"]
    upstream = dict(cell=T.dY_cell, net=T.dY_net)
    say("large: oracle.spmm_bwd on the three whole transposed relations")
    with ThreadPoolExecutor(max_workers=3) as pool:
        futs = {name: pool.submit(oracle.spmm_bwd, *tr[name], upstream[dst], whole[f"idx_{src}"], True)
                for name, src, dst in RELATIONS}
        for name, src, dst in RELATIONS:
            At = P.device_transpose(inputs["dev_rel"][name])
            idx = dev(whole[f"idx_{src}"].astype(np.uint16).view(np.int16))
            G = torch.full((At.n_rows, K), float("nan"), dtype=torch.float32, device="cuda")
            say(f"large: dr_spmm_bwd.{name}, {At.nnz} edges")
            P.dr_spmm_bwd(At, inputs["dT"][f"dY_{dst}"], idx, D, K, G)
            torch.cuda.synchronize()
            want, l1row, l1elem = futs[name].result()
            got = G.cpu().numpy()
            worst = assert_row_bound(got, want, l1row, f"G_{name}")
            assert_elem_bound(got, want, l1elem, f"G_{name}")
            if name == "near":
                # the same gradient from the kernel that stages the dH rows of a placement tile in LDS
                plan = P.SpmmPlan(At, D, dev(inputs["g"].cell_order))
                n_tiles, reuse = plan.dr_spmm_plan_info()
                Gp = torch.full((At.n_rows, K), float("nan"), dtype=torch.float32, device="cuda")
                plan.dr_spmm_bwd_planned(inputs["dT"][f"dY_{dst}"], idx, K, Gp)
                torch.cuda.synchronize()
                gp = Gp.cpu().numpy()
                worst_p = assert_row_bound(gp, want, l1row, "G_near (planned)")
                assert_elem_bound(gp, want, l1elem, "G_near (planned)")
                say(f"   dr_spmm_bwd_planned.near: {n_tiles} tiles, reuse {reuse:.2f}, worst err / row L1 = {worst_p:.2e}")
                plan.dr_spmm_plan_destroy()
            # accumulate: a second pass onto the first doubles every element exactly
            P.dr_spmm_bwd(At, inputs["dT"][f"dY_{dst}"], idx, D, K, G, accumulate=True)
            torch.cuda.synchronize()
            assert np.array_equal(G.cpu().numpy(), got + got), f"G_{name} accumulate"
            say(f"   {got.shape[0]} rows x {K}: worst err / row L1 = {worst:.2e}")


@pytest.mark.parametrize("k", (8, 16, 64))
def test_other_widths_of_the_k_sweep_on_the_cells_and_near(inputs, k):
    """The other widths bench.py's k sweep times (other kernel instantiations): dr_topk of all cells bit-exact, and
    every element of dr_spmm_fwd, dr_spmm_bwd and dr_spmm_bwd_planned on the whole `near` relation."""
    D, T, tr = inputs["D"], inputs["T"], inputs["tr"]
    rel = inputs["rel"]["near"]
    say(f"large k={k}: oracle.topk of the cells, oracle.spmm_fwd / spmm_bwd of near")
    with ThreadPoolExecutor(max_workers=2) as pool:
        ov, oi = oracle.topk(T.X_cell, k)
        f_fwd = pool.submit(oracle.spmm_fwd, rel.rowptr, rel.colidx, rel.vals, ov, oi, D, True)
        f_bwd = pool.submit(oracle.spmm_bwd, *tr["near"], T.dY_cell, oi, True)
        X = inputs["dT"]["X_cell"]
        vals = torch.full((X.shape[0], k), float("nan"), dtype=torch.float32, device="cuda")
        idx = torch.full((X.shape[0], k), -1, dtype=torch.int16, device="cuda")
        P.dr_topk(X, k, vals, idx)
        torch.cuda.synchronize()
        assert np.array_equal(host_idx(idx), oi)
        assert np.array_equal(vals.cpu().numpy().astype(np.float64), ov)
        A = inputs["dev_rel"]["near"]
        H = torch.full((A.n_rows, D), float("nan"), dtype=torch.float32, device="cuda")
        P.dr_spmm_fwd(A, vals, idx, D, k, H)
        torch.cuda.synchronize()
        want, l1row, l1elem = f_fwd.result()
        worst_f = assert_row_bound(H.cpu().numpy(), want, l1row, f"H_near k={k}")
        assert_elem_bound(H.cpu().numpy(), want, l1elem, f"H_near k={k}")
        del want, l1row, l1elem, H
        At = P.device_transpose(A)
        want, l1row, l1elem = f_bwd.result()
        G = torch.full((At.n_rows, k), float("nan"), dtype=torch.float32, device="cuda")
        P.dr_spmm_bwd(At, inputs["dT"]["dY_cell"], idx, D, k, G)
        plan = P.SpmmPlan(At, D, dev(inputs["g"].cell_order))
        Gp = torch.full((At.n_rows, k), float("nan"), dtype=torch.float32, device="cuda")
        plan.dr_spmm_bwd_planned(inputs["dT"]["dY_cell"], idx, k, Gp)
        torch.cuda.synchronize()
        worst_b = assert_row_bound(G.cpu().numpy(), want, l1row, f"G_near k={k}")
        assert_elem_bound(G.cpu().numpy(), want, l1elem, f"G_near k={k}")
        worst_p = assert_row_bound(Gp.cpu().numpy(), want, l1row, f"G_near (planned) k={k}")
        assert_elem_bound(Gp.cpu().numpy(), want, l1elem, f"G_near (planned) k={k}")
        plan.dr_spmm_plan_destroy()
    say(f"   worst err / row L1: fwd {worst_f:.2e}, bwd {worst_b:.2e}, bwd planned {worst_p:.2e}")
