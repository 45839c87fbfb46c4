"""Sampled parity checks at sizes the oracle cannot recompute whole: the HIP layer runs on the whole graph,
the oracle recomputes a random sample of output rows one by one from induced sub-problems (every edge of the
sampled rows, exact full-graph edge values).  Used by the large- and medium-configuration test modules."""
import numpy as np
import torch

import oracle
import paper_2508_16769_amd as P
from circuit_synth import make_graph, make_tensors, workload
from gpu_util import dev, host_idx, say

ROW_TOL = 1e-4


def sub_rows(rel, rows):
    """Induced sub-problem: the given destination rows with all their edges; returns (rowptr, local colidx,
    vals, unique source ids)."""
    rp = rel.rowptr.astype(np.int64)
    deg = rp[rows + 1] - rp[rows]
    sub_rp = np.zeros(len(rows) + 1, np.int32)
    sub_rp[1:] = np.cumsum(deg)
    take = np.concatenate([np.arange(rp[r], rp[r + 1]) for r in rows]) if len(rows) else np.zeros(0, np.int64)
    cols = rel.colidx[take]
    uniq, local = np.unique(cols, return_inverse=True)
    return sub_rp, local.astype(np.int32), rel.vals[take], uniq


def oracle_forward_rows(rel, rows, X_src, k, D):
    """H[rows] of one relation, plus the per-element L1 of its terms."""
    sub_rp, local, vals, uniq = sub_rows(rel, rows)
    ov, oi = oracle.topk(X_src[uniq], k)
    H, _, l1 = oracle.spmm_fwd(sub_rp, local, vals, ov, oi, D, want_l1elem=True)
    return H, l1


def make_inputs(name):
    """Graph, tensors, oracle relations and transposes, device copies for one workload."""
    w = workload(name)
    say(f"{name}: generating graph and tensors")
    g = make_graph(name, seed=0)
    T = make_tensors(g.Nc, g.Nn, w["D"], seed=0)
    say(f"{name}: device setup")
    dev_rel = dict(near=P.device_relation(g.near, P.DR_NORM_MEAN), pins=P.device_relation(g.pins, P.DR_NORM_MEAN),
                   pinned=P.device_relation(g.pinned, P.DR_NORM_SYM))
    say(f"{name}: oracle edge values and transposes")
    rel = dict(near=oracle.relation(g.near, oracle.NORM_MEAN), pins=oracle.relation(g.pins, oracle.NORM_MEAN),
               pinned=oracle.relation(g.pinned, oracle.NORM_SYM))
    tr = {n: oracle.csr_transpose(rel[n].M, rel[n].N, rel[n].rowptr, rel[n].colidx, rel[n].vals) for n in rel}
    dT = dict(X_cell=dev(T.X_cell), X_net=dev(T.X_net), dY_cell=dev(T.dY_cell), dY_net=dev(T.dY_net),
              W={n: dev(T.W[n]) for n in P.WEIGHT_NAMES})
    return dict(name=name, g=g, T=T, D=w["D"], k_default=w["k"], rel=rel, tr=tr, dev_rel=dev_rel, dT=dT)


def run_layer(li, k):
    """One heteroconv_fwd + heteroconv_bwd on the whole graph; returns the inputs plus every output."""
    g, D, dT = li["g"], li["D"], li["dT"]
    layer = P.HeteroConv(li["dev_rel"]["near"], li["dev_rel"]["pins"], li["dev_rel"]["pinned"], D, k, k)
    saved = layer.alloc_saved()
    Y_cell = torch.empty((g.Nc, D), dtype=torch.float32, device="cuda")
    Y_net = torch.empty((g.Nn, D), dtype=torch.float32, device="cuda")
    dX_cell, dX_net = torch.empty_like(Y_cell), torch.empty_like(Y_net)
    dW = {n: torch.empty((D, D), dtype=torch.float32, device="cuda") for n in P.WEIGHT_NAMES}
    say(f"{li['name']} k={k}: heteroconv_fwd + heteroconv_bwd")
    layer.heteroconv_fwd(dT["X_cell"], dT["X_net"], dT["W"], Y_cell, Y_net, saved)
    layer.heteroconv_bwd(dT["dY_cell"], dT["dY_net"], dT["W"], saved, dX_cell, dX_net, dW)
    torch.cuda.synchronize()
    return dict(li, k=k, saved=saved, Y_cell=Y_cell, Y_net=Y_net, dX_cell=dX_cell, dX_net=dX_net, dW=dW, layer=layer)


def check_setup(r):
    for name in ("near", "pins", "pinned"):
        say(f"{r['name']}.{name}: edge values")
        assert np.array_equal(r["dev_rel"][name].vals.cpu().numpy().view(np.uint32), r["rel"][name].vals.view(np.uint32))
    # transposes held by the context, compared on sampled rows of A^T through a backward SpMM below; here the
    # row pointers of a device transpose are checked in full (integer-exact)
    At = P.device_transpose(r["dev_rel"]["pins"])
    o_rp, o_ci, o_v = r["tr"]["pins"]
    assert np.array_equal(At.rowptr.cpu().numpy(), o_rp)
    assert np.array_equal(At.colidx.cpu().numpy(), o_ci)
    assert np.array_equal(At.vals.cpu().numpy().view(np.uint32), o_v.view(np.uint32))


def check_forward(r):
    g, T, D, k, rel = r["g"], r["T"], r["D"], r["k"], r["rel"]
    rng = np.random.default_rng(123)
    Xc, Xn = T.X_cell, T.X_net
    W = {n: T.W[n].astype(np.float64) for n in T.W}

    # top-k on sampled rows: bit-exact
    for name, X, key in (("cell", Xc, "cell"), ("net", Xn, "net")):
        rows = np.sort(rng.choice(X.shape[0], 3000, replace=False))
        ov, oi = oracle.topk(X[rows], k)
        gi = host_idx(r["saved"][f"idx_{key}"][torch.from_numpy(rows).cuda()])
        gv = r["saved"][f"vals_{key}"][torch.from_numpy(rows).cuda()].cpu().numpy()
        assert np.array_equal(gi, oi), name
        assert np.array_equal(gv.astype(np.float64), ov), name

    # cell outputs: sampled rows plus every high-degree near row among a random window
    deg_pins = np.diff(rel["pins"].rowptr)
    cells = np.sort(rng.choice(g.Nc, 400, replace=False))
    nets = np.unique(np.concatenate([rng.choice(g.Nn, 300, replace=False), np.argsort(-deg_pins)[:3]]))
    say(f"{r['name']}: forward on {len(cells)} sampled cells and {len(nets)} nets (max net degree {deg_pins[nets].max()})")
    ovc, oic = oracle.topk(Xc[cells], k)
    Xs_c = oracle.densify(ovc, oic, D)
    Hn, l1n = oracle_forward_rows(rel["near"], cells, Xc, k, D)
    Hq, l1q = oracle_forward_rows(rel["pinned"], cells, Xn, k, D)
    Zn = Xs_c @ W["self_near"] + Hn @ W["neigh_near"]
    Zq = Hq @ W["pinned"]
    L1n = np.abs(Xs_c) @ np.abs(W["self_near"]) + l1n @ np.abs(W["neigh_near"])
    L1q = l1q @ np.abs(W["pinned"])
    sel = torch.from_numpy(cells).cuda()
    for nm, want, l1 in (("H_near", Hn, l1n), ("H_pinned", Hq, l1q)):
        got = r["saved"][nm][sel].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - want).max(axis=1) <= ROW_TOL * l1.sum(axis=1) + 1e-30), nm
        assert np.all(np.abs(got - want) <= 1e-5 * l1 + 1e-30), nm
    Yc = r["Y_cell"][sel].cpu().numpy().astype(np.float64)
    L1 = np.maximum(L1n, L1q)
    assert np.all(np.abs(Yc - np.maximum(Zn, Zq)).max(axis=1) <= ROW_TOL * L1.sum(axis=1))
    mask = r["saved"]["mask"][sel].cpu().numpy()
    decided = np.abs(Zn - Zq) > 2e-5 * L1
    assert decided.mean() > 0.99
    assert np.array_equal(mask[decided], (Zn >= Zq)[decided].astype(np.uint8))

    ovn, oin = oracle.topk(Xn[nets], k)
    Xs_n = oracle.densify(ovn, oin, D)
    Hp, l1p = oracle_forward_rows(rel["pins"], nets, Xc, k, D)
    Yn = Xs_n @ W["self_pins"] + Hp @ W["neigh_pins"]
    L1p = np.abs(Xs_n) @ np.abs(W["self_pins"]) + l1p @ np.abs(W["neigh_pins"])
    seln = torch.from_numpy(nets).cuda()
    got = r["saved"]["H_pins"][seln].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - Hp).max(axis=1) <= ROW_TOL * l1p.sum(axis=1) + 1e-30)
    assert np.all(np.abs(got - Hp) <= 1e-5 * l1p + 1e-30)          # includes the 2000-edge nets
    got = r["Y_net"][seln].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - Yn).max(axis=1) <= ROW_TOL * L1p.sum(axis=1))


def check_backward(r):
    """dX of sampled source rows, recomputed by the oracle from the two-hop neighbourhood (the destinations of
    the sampled sources need their own forward to decide the max-merge mask)."""
    g, T, D, k, rel = r["g"], r["T"], r["D"], r["k"], r["rel"]
    rng = np.random.default_rng(321)
    Xc, Xn = T.X_cell, T.X_net
    W = {n: T.W[n].astype(np.float64) for n in T.W}
    tr = r["tr"]

    def t_rows(name, rows):          # rows of A^T: (sub rowptr, destination ids, values)
        rp, ci, v = tr[name]
        rp = rp.astype(np.int64)
        take = np.concatenate([np.arange(rp[j], rp[j + 1]) for j in rows])
        sub = np.zeros(len(rows) + 1, np.int64)
        sub[1:] = np.cumsum(rp[rows + 1] - rp[rows])
        return sub, ci[take], v[take].astype(np.float64)

    def masks_for(cells):            # oracle forward of the given cells -> (mask, decided)
        ovc, oic = oracle.topk(Xc[cells], k)
        Xs_c = oracle.densify(ovc, oic, D)
        Hn, l1n = oracle_forward_rows(rel["near"], cells, Xc, k, D)
        Hq, l1q = oracle_forward_rows(rel["pinned"], cells, Xn, k, D)
        Zn = Xs_c @ W["self_near"] + Hn @ W["neigh_near"]
        Zq = Hq @ W["pinned"]
        L1 = np.maximum(np.abs(Xs_c) @ np.abs(W["self_near"]) + l1n @ np.abs(W["neigh_near"]), l1q @ np.abs(W["pinned"]))
        return (Zn >= Zq), np.abs(Zn - Zq) > 2e-5 * L1

    # ---- cells as sources: near^T and pins^T plus the self term ----
    src = np.sort(rng.choice(g.Nc, 60, replace=False))
    s_near, d_near, a_near = t_rows("near", src)
    s_pins, d_pins, a_pins = t_rows("pins", src)
    need = np.unique(np.concatenate([src, d_near]))                     # cells whose mask is needed
    say(f"{r['name']}: backward on {len(src)} cells (needs the forward of {len(need)} cells)")
    m_need, dec_need = masks_for(need)
    gm = r["saved"]["mask"][torch.from_numpy(need).cuda()].cpu().numpy().astype(bool)
    assert np.array_equal(gm[dec_need], m_need[dec_need])
    pos = {int(c): i for i, c in enumerate(need)}
    _, idx_src = oracle.topk(Xc[src], k)
    dYc = T.dY_cell.astype(np.float64)
    dYn = T.dY_net.astype(np.float64)
    got = r["dX_cell"][torch.from_numpy(src).cuda()].cpu().numpy().astype(np.float64)
    checked = 0
    for q, j in enumerate(src):
        dsts = d_near[s_near[q]:s_near[q + 1]]
        rows_m = np.array([pos[int(i)] for i in dsts] + [pos[int(j)]], dtype=np.int64)
        if not dec_need[rows_m].all():
            continue                                                    # a neighbour's merge is a numerical tie
        cols = idx_src[q].astype(np.int64)
        dZ = np.where(m_need[rows_m[:-1]], dYc[dsts], 0.0)
        dH = dZ @ W["neigh_near"].T
        terms = a_near[s_near[q]:s_near[q + 1], None] * dH[:, cols]
        nets_j = d_pins[s_pins[q]:s_pins[q + 1]]
        dHp = dYn[nets_j] @ W["neigh_pins"].T
        terms_p = a_pins[s_pins[q]:s_pins[q + 1], None] * dHp[:, cols]
        self_t = (np.where(m_need[rows_m[-1]], dYc[j], 0.0) @ W["self_near"].T)[cols]
        want = terms.sum(axis=0) + terms_p.sum(axis=0) + self_t
        l1 = np.abs(terms).sum() + np.abs(terms_p).sum() + np.abs(self_t).sum()
        assert np.abs(got[q][cols] - want).max() <= ROW_TOL * l1, (j, np.abs(got[q][cols] - want).max(), l1)
        off = np.ones(D, bool)
        off[cols] = False
        assert np.all(got[q][off] == 0)
        checked += 1
    assert checked >= 30

    # ---- nets as sources: pinned^T plus the pins self term; include the highest-fanout nets ----
    deg_t = np.diff(tr["pinned"][0])
    srcn = np.unique(np.concatenate([rng.choice(g.Nn, 40, replace=False), np.argsort(-deg_t)[:2]]))
    s_q, d_q, a_q = t_rows("pinned", srcn)
    need = np.unique(d_q)
    say(f"{r['name']}: backward on {len(srcn)} nets (max fan-out {deg_t[srcn].max()}, forward of {len(need)} cells)")
    m_need, dec_need = masks_for(need)
    pos = {int(c): i for i, c in enumerate(need)}
    _, idx_n = oracle.topk(Xn[srcn], k)
    got = r["dX_net"][torch.from_numpy(srcn).cuda()].cpu().numpy().astype(np.float64)
    checked = 0
    for q, j in enumerate(srcn):
        dsts = d_q[s_q[q]:s_q[q + 1]]
        rows_m = np.array([pos[int(i)] for i in dsts], dtype=np.int64)
        if not dec_need[rows_m].all():
            continue
        cols = idx_n[q].astype(np.int64)
        dZ = np.where(m_need[rows_m], 0.0, dYc[dsts])                   # the pinned branch gets (1 - M) * dY
        dH = dZ @ W["pinned"].T
        terms = a_q[s_q[q]:s_q[q + 1], None] * dH[:, cols]
        self_t = (dYn[j] @ W["self_pins"].T)[cols]
        want = terms.sum(axis=0) + self_t
        l1 = np.abs(terms).sum() + np.abs(self_t).sum()
        assert np.abs(got[q][cols] - want).max() <= ROW_TOL * l1, (j, len(dsts))
        checked += 1
    assert checked >= 20


def check_weight_gradients(r):
    """dW is a reduction over all rows, so single outputs cannot be sampled; it is checked through an identity
    that holds at any size: for a random probe P, sum(dW_neigh_pins * P) == sum_i (H_pins[i] P) . dY_net[i],
    with the right-hand side evaluated in fp64 on the host from the saved H_pins."""
    T, D = r["T"], r["D"]
    rng = np.random.default_rng(9)
    Pm = rng.standard_normal((D, D))
    H = r["saved"]["H_pins"].cpu().numpy().astype(np.float64)
    dYn = T.dY_net.astype(np.float64)
    want = float(np.sum((H @ Pm) * dYn))
    l1 = float(np.sum(np.abs(H) @ np.abs(Pm) * np.abs(dYn)))
    got = float(np.sum(r["dW"]["neigh_pins"].cpu().numpy().astype(np.float64) * Pm))
    assert abs(got - want) <= 1e-5 * l1, (got, want, l1)
