"""Parity checks at sizes where the oracle cannot recompute the whole layer in seconds: the HIP layer runs on the
whole graph, and the expected values come from `oracle/` run on an induced sub-problem -- the sampled nodes plus
everything that reaches them (every edge of the rows involved, the full graph's edge values) -- so each compared
output is what the oracle's layer forward / backward computes for that node.  Weight gradients are reductions over
all rows: they are checked entry by entry as fp64 dot products over all rows and through a probe identity.
Used by the large- and medium-configuration test modules."""
import numpy as np
import torch

import oracle
import paper_2508_16769_amd as P
from circuit_synth import make_graph, make_tensors, workload
from gpu_util import dev, host_idx, say

ROW_TOL = 1e-4
ELEM_TOL = 1e-5

_INPUTS = {}


def make_inputs(name):
    """Graph, tensors, oracle relations and transposes, device copies for one workload (built once per process)."""
    if name in _INPUTS:
        return _INPUTS[name]
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
    _INPUTS[name] = dict(name=name, g=g, T=T, D=w["D"], k_default=w["k"], rel=rel, tr=tr, dev_rel=dev_rel, dT=dT,
                         whole={})
    return _INPUTS[name]


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
    for name in ("near", "pins", "pinned"):
        say(f"{r['name']}.{name}: device transpose, every entry")
        At = P.device_transpose(r["dev_rel"][name])
        o_rp, o_ci, o_v = r["tr"][name]
        assert np.array_equal(At.rowptr.cpu().numpy(), o_rp)
        assert np.array_equal(At.colidx.cpu().numpy(), o_ci)
        assert np.array_equal(At.vals.cpu().numpy().view(np.uint32), o_v.view(np.uint32))


# ----------------------------------------------------------------------------------------------------------
# induced sub-problems
# ----------------------------------------------------------------------------------------------------------

def _rows_cols(rowptr, colidx, rows):
    """Concatenated column ids of the given CSR rows."""
    rp = rowptr.astype(np.int64)
    if len(rows) == 0:
        return np.zeros(0, np.int64)
    return np.concatenate([colidx[rp[r]:rp[r + 1]] for r in rows]).astype(np.int64)


def sub_rows(rel, rows):
    """The given destination rows of one relation with all their edges: (rowptr, local colidx, vals, unique source ids)."""
    rp = rel.rowptr.astype(np.int64)
    deg = rp[rows + 1] - rp[rows]
    sub_rp = np.zeros(len(rows) + 1, np.int32)
    sub_rp[1:] = np.cumsum(deg)
    take = np.concatenate([np.arange(rp[r], rp[r + 1]) for r in rows]) if len(rows) else np.zeros(0, np.int64)
    cols = rel.colidx[take]
    uniq, local = np.unique(cols, return_inverse=True)
    return sub_rp, local.astype(np.int32), rel.vals[take], uniq


def _sub_csr(relation, rows_global, full_rows, col_ids, n_rows):
    """CSR over local ids: local row q (= rows_global[q]) keeps its edges if it is in `full_rows` (a boolean over
    local rows) -- only those whose source is in col_ids (sorted global ids; for a row that must be exact all of them
    are) -- with the full graph's edge values."""
    rp = relation.rowptr.astype(np.int64)
    out_rp = np.zeros(n_rows + 1, np.int64)
    cols, vals = [], []
    for q, r in enumerate(rows_global):
        if full_rows[q]:
            c = relation.colidx[rp[r]:rp[r + 1]].astype(np.int64)
            v = relation.vals[rp[r]:rp[r + 1]]
            pos = np.searchsorted(col_ids, c)
            ok = (pos < len(col_ids)) & (col_ids[np.minimum(pos, len(col_ids) - 1)] == c)
            cols.append(pos[ok])
            vals.append(v[ok])
            out_rp[q + 1] = int(ok.sum())
    np.cumsum(out_rp, out=out_rp)
    ci = np.concatenate(cols).astype(np.int32) if cols else np.zeros(0, np.int32)
    va = np.concatenate(vals).astype(np.float32) if vals else np.zeros(0, np.float32)
    return oracle.Relation(n_rows, len(col_ids), out_rp.astype(np.int32), ci, va)


def induced_problem(r, cells_exact, nets_exact, cells_src=(), nets_src=()):
    """The sub-problem on which the oracle's layer gives, for the cells / nets in *_exact, the forward outputs of the
    whole graph, and for the cells / nets in *_src the input gradients of the whole graph.  The caller makes
    cells_exact contain every cell whose merge mask the wanted gradients depend on (the sources themselves, their
    `near` destinations, the member cells of nets_src)."""
    rel = r["rel"]
    cells_exact = np.unique(np.asarray(cells_exact, np.int64))
    nets_exact = np.unique(np.asarray(nets_exact, np.int64))
    cells_src = np.unique(np.asarray(cells_src, np.int64))
    nets_src = np.unique(np.asarray(nets_src, np.int64))
    C = np.unique(np.concatenate([cells_exact, cells_src,
                                  _rows_cols(rel["near"].rowptr, rel["near"].colidx, cells_exact),
                                  _rows_cols(rel["pins"].rowptr, rel["pins"].colidx, nets_exact)]))
    pins_t = r["tr"]["pins"]          # rows = cells, columns = the nets a cell pins
    N = np.unique(np.concatenate([nets_exact, nets_src,
                                  _rows_cols(rel["pinned"].rowptr, rel["pinned"].colidx, cells_exact),
                                  _rows_cols(pins_t[0], pins_t[1], cells_src)]))
    cell_full = np.isin(C, cells_exact)
    near = _sub_csr(rel["near"], C, cell_full, C, len(C))
    pinned = _sub_csr(rel["pinned"], C, cell_full, N, len(C))
    pins = _sub_csr(rel["pins"], N, np.ones(len(N), bool), C, len(N))     # members outside C are dropped
    return dict(C=C, N=N, near=near, pins=pins, pinned=pinned,
                loc_cell=lambda ids: np.searchsorted(C, ids), loc_net=lambda ids: np.searchsorted(N, ids))


def _gpu_rows(t, rows):
    return t[torch.from_numpy(np.asarray(rows, np.int64)).cuda()].cpu().numpy()


def check_topk_sampled(r, n_rows=3000):
    """D-ReLU outputs of sampled rows of both node types, bit-exact."""
    T, k = r["T"], r["k"]
    rng = np.random.default_rng(123)
    for key, X in (("cell", T.X_cell), ("net", T.X_net)):
        rows = np.sort(rng.choice(X.shape[0], min(n_rows, X.shape[0]), replace=False))
        ov, oi = oracle.topk(X[rows], k)
        assert np.array_equal(host_idx(r["saved"][f"idx_{key}"][torch.from_numpy(rows).cuda()]), oi), key
        assert np.array_equal(_gpu_rows(r["saved"][f"vals_{key}"], rows).astype(np.float64), ov), key


def check_forward(r):
    """Layer outputs, aggregated messages and merge mask of sampled cells and nets against oracle.heteroconv_fwd on
    the induced sub-problem."""
    g, T, D, k, rel = r["g"], r["T"], r["D"], r["k"], r["rel"]
    check_topk_sampled(r)
    rng = np.random.default_rng(123)
    deg_pins = np.diff(rel["pins"].rowptr)
    deg_near = np.diff(rel["near"].rowptr)
    cells = np.unique(np.concatenate([rng.choice(g.Nc, 400, replace=False), np.argsort(-deg_near)[:3]]))
    nets = np.unique(np.concatenate([rng.choice(g.Nn, 300, replace=False), np.argsort(-deg_pins)[:3]]))
    sp = induced_problem(r, cells, nets)
    say(f"{r['name']} k={k}: forward of {len(cells)} cells (max near degree {deg_near[cells].max()}) and {len(nets)} nets "
        f"(max degree {deg_pins[nets].max()}); oracle sub-problem {len(sp['C'])} cells, {len(sp['N'])} nets")
    of = oracle.heteroconv_fwd(sp["near"], sp["pins"], sp["pinned"], T.X_cell[sp["C"]], T.X_net[sp["N"]], T.W, k, k)
    lc, ln = sp["loc_cell"](cells), sp["loc_net"](nets)

    # aggregated messages saved by the layer: oracle.spmm_fwd on the sub-problem's relations gives the same rows as the
    # layer oracle plus the L1 norm of the terms of every element
    for nm, sub, key, loc, rows in (("H_near", sp["near"], "cell", lc, cells), ("H_pinned", sp["pinned"], "net", lc, cells),
                                    ("H_pins", sp["pins"], "cell", ln, nets)):
        want, l1row, l1 = oracle.spmm_fwd(sub.rowptr, sub.colidx, sub.vals, of[f"vals_{key}"], of[f"idx_{key}"], D, want_l1elem=True)
        assert np.array_equal(want[loc], of[nm][loc])
        got = _gpu_rows(r["saved"][nm], rows).astype(np.float64)
        assert np.all(np.abs(got - want[loc]).max(axis=1) <= ROW_TOL * l1row[loc] + 1e-30), nm
        assert np.all(np.abs(got - want[loc]) <= ELEM_TOL * l1[loc] + 1e-30), nm
    l1c, l1n = of["l1_cell"][lc], of["l1_net"][ln]
    Yc = _gpu_rows(r["Y_cell"], cells).astype(np.float64)
    assert np.all(np.abs(Yc - of["Y_cell"][lc]).max(axis=1) <= ROW_TOL * l1c.sum(axis=1))
    assert np.all(np.abs(Yc - of["Y_cell"][lc]) <= ELEM_TOL * l1c + 1e-30)
    Yn = _gpu_rows(r["Y_net"], nets).astype(np.float64)
    assert np.all(np.abs(Yn - of["Y_net"][ln]).max(axis=1) <= ROW_TOL * l1n.sum(axis=1))
    assert np.all(np.abs(Yn - of["Y_net"][ln]) <= ELEM_TOL * l1n + 1e-30)
    mask = _gpu_rows(r["saved"]["mask"], cells)
    assert set(np.unique(mask)) <= {0, 1}
    decided = np.abs(of["Z_near"][lc] - of["Z_pinned"][lc]) > 2e-5 * l1c
    assert decided.mean() > 0.99
    assert np.array_equal(mask[decided], of["mask"][lc][decided])


def check_backward(r):
    """dX of sampled source cells and nets against oracle.heteroconv_bwd on the induced sub-problem (the sampled
    sources, every destination they feed, and the forward of those destinations, which decides their merge mask).
    The max-merge mask is a floating-point decision: the GPU's must equal the oracle's wherever the two branches are
    separated by more than the error bound; the oracle's backward then runs on the GPU's mask for those cells, so
    that numerical ties route the gradient the same way on both sides and every sampled source is compared."""
    g, T, D, k, rel, tr = r["g"], r["T"], r["D"], r["k"], r["rel"], r["tr"]
    rng = np.random.default_rng(321)
    deg_t = np.diff(tr["pinned"][0])
    src_c = np.sort(rng.choice(g.Nc, 60, replace=False))
    src_n = np.unique(np.concatenate([rng.choice(g.Nn, 40, replace=False), np.argsort(-deg_t)[:1]]))
    need_mask = np.unique(np.concatenate([src_c, _rows_cols(tr["near"][0], tr["near"][1], src_c),
                                          _rows_cols(tr["pinned"][0], tr["pinned"][1], src_n)]))
    sp = induced_problem(r, need_mask, [], src_c, src_n)
    say(f"{r['name']} k={k}: backward of {len(src_c)} cells and {len(src_n)} nets (max fan-out {deg_t[src_n].max()}); "
        f"masks of {len(need_mask)} cells; oracle sub-problem {len(sp['C'])} cells, {len(sp['N'])} nets")
    of = oracle.heteroconv_fwd(sp["near"], sp["pins"], sp["pinned"], T.X_cell[sp["C"]], T.X_net[sp["N"]], T.W, k, k)
    lm = sp["loc_cell"](need_mask)
    gm = _gpu_rows(r["saved"]["mask"], need_mask)
    decided = np.abs(of["Z_near"][lm] - of["Z_pinned"][lm]) > 2e-5 * of["l1_cell"][lm]
    assert decided.mean() > 0.99
    assert np.array_equal(gm[decided], of["mask"][lm][decided])
    of["mask"][lm] = gm
    ob = oracle.heteroconv_bwd(sp["near"], sp["pins"], sp["pinned"], T.W, of, T.dY_cell[sp["C"]], T.dY_net[sp["N"]])

    for key, src, loc, dX in (("cell", src_c, sp["loc_cell"](src_c), r["dX_cell"]), ("net", src_n, sp["loc_net"](src_n), r["dX_net"])):
        idx = of[f"idx_{key}"][loc].astype(np.int64)
        assert np.array_equal(host_idx(r["saved"][f"idx_{key}"][torch.from_numpy(src).cuda()]), idx)
        got = _gpu_rows(dX, src).astype(np.float64)
        want, l1 = ob[f"dXs_{key}"][loc], ob[f"l1_dxs_{key}"][loc]
        err = np.abs(np.take_along_axis(got, idx, axis=1) - want)
        assert np.all(err.max(axis=1) <= ROW_TOL * l1.sum(axis=1)), (key, float((err.max(axis=1) / l1.sum(axis=1)).max()))
        off = np.ones_like(got, bool)
        np.put_along_axis(off, idx, False, axis=1)
        assert np.all(got[off] == 0), key
        say(f"   dX_{key}: {len(src)} rows compared, worst err / row L1 = {float((err.max(axis=1) / l1.sum(axis=1)).max()):.2e}")


# ----------------------------------------------------------------------------------------------------------
# weight gradients
# ----------------------------------------------------------------------------------------------------------

def whole_forward_state(r):
    """Operands of the five weight gradients for every row: the D-ReLU outputs (dense) and the aggregated messages.
    At the workload's own k they are the oracle's, computed on the whole graph (oracle.topk, oracle.spmm_fwd; kept
    for the other tests of the process); at the other k of a sweep they are the layer's saved arrays, whose rows the
    forward check samples."""
    T, D, k, rel = r["T"], r["D"], r["k"], r["rel"]
    if k == r["k_default"]:
        w = oracle_whole(r, k)
        return dict(Xs_cell=oracle.densify(w["vals_cell"], w["idx_cell"], D), Xs_net=oracle.densify(w["vals_net"], w["idx_net"], D),
                    H_near=w["H_near"][0], H_pins=w["H_pins"][0], H_pinned=w["H_pinned"][0], source="oracle on the whole graph")
    s = r["saved"]
    f64 = lambda t: t.cpu().numpy().astype(np.float64)
    return dict(Xs_cell=oracle.densify(f64(s["vals_cell"]), host_idx(s["idx_cell"]), D),
                Xs_net=oracle.densify(f64(s["vals_net"]), host_idx(s["idx_net"]), D),
                H_near=f64(s["H_near"]), H_pins=f64(s["H_pins"]), H_pinned=f64(s["H_pinned"]), source="the layer's saved arrays")


def oracle_whole(li, k):
    """oracle.topk of both node types and oracle.spmm_fwd of the three relations on the whole graph (independent
    calls side by side on the host's cores; each call is the single-threaded oracle)."""
    key = ("fwd", k)
    if key in li["whole"]:
        return li["whole"][key]
    from concurrent.futures import ThreadPoolExecutor
    T, D, rel = li["T"], li["D"], li["rel"]
    say(f"{li['name']} k={k}: oracle.topk and oracle.spmm_fwd on the whole graph")
    with ThreadPoolExecutor(max_workers=5) as pool:
        fc = pool.submit(oracle.topk, T.X_cell, k)
        fn = pool.submit(oracle.topk, T.X_net, k)
        vc, ic = fc.result()
        f1 = pool.submit(oracle.spmm_fwd, rel["near"].rowptr, rel["near"].colidx, rel["near"].vals, vc, ic, D, True)
        f2 = pool.submit(oracle.spmm_fwd, rel["pins"].rowptr, rel["pins"].colidx, rel["pins"].vals, vc, ic, D, True)
        vn, inn = fn.result()
        f3 = pool.submit(oracle.spmm_fwd, rel["pinned"].rowptr, rel["pinned"].colidx, rel["pinned"].vals, vn, inn, D, True)
        out = dict(vals_cell=vc, idx_cell=ic, vals_net=vn, idx_net=inn, H_near=f1.result(), H_pins=f2.result(), H_pinned=f3.result())
    li["whole"][key] = out
    return out


def check_weight_gradients(r, n_entries=64):
    """All five weight gradients, each through (a) n_entries sampled entries dW[a,b] = sum_i A[i,a] B[i,b] evaluated as
    fp64 dot products over all rows, bound 1e-4 x the L1 norm of that entry's terms, and (b) the probe identity
    sum(dW * P) = sum_i (A[i] P) . B[i] for a random P.  A = the module's forward operand (see whole_forward_state),
    B = the upstream gradient routed by the layer's saved merge mask."""
    T, D = r["T"], r["D"]
    st = whole_forward_state(r)
    say(f"{r['name']} k={r['k']}: five weight gradients, operands from {st['source']}")
    mask = r["saved"]["mask"].cpu().numpy()
    dYc, dYn = T.dY_cell.astype(np.float64), T.dY_net.astype(np.float64)
    dZn, dZq = np.where(mask == 1, dYc, 0.0), np.where(mask == 0, dYc, 0.0)
    ops = dict(self_near=(st["Xs_cell"], dZn), neigh_near=(st["H_near"], dZn), self_pins=(st["Xs_net"], dYn),
               neigh_pins=(st["H_pins"], dYn), pinned=(st["H_pinned"], dZq))
    rng = np.random.default_rng(9)
    for name in P.WEIGHT_NAMES:
        A, B = ops[name]
        got = r["dW"][name].cpu().numpy().astype(np.float64)
        ea, eb = rng.integers(0, D, n_entries), rng.integers(0, D, n_entries)
        worst = 0.0
        for a, b in zip(ea, eb):
            terms = A[:, a] * B[:, b]
            want, l1 = float(terms.sum()), float(np.abs(terms).sum())
            assert abs(got[a, b] - want) <= ROW_TOL * l1, (name, int(a), int(b), got[a, b], want, l1)
            worst = max(worst, abs(got[a, b] - want) / l1)
        Pm = rng.standard_normal((D, D))
        want = float(np.sum((A @ Pm) * B))
        l1 = float(np.sum((np.abs(A) @ np.abs(Pm)) * np.abs(B)))
        assert abs(float(np.sum(got * Pm)) - want) <= 1e-5 * l1, (name, "probe identity")
        say(f"   dW.{name}: {n_entries} entries, worst err / entry L1 = {worst:.2e}; probe identity holds")
