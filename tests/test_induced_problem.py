"""Host-side check of the sub-problem construction the full-size parity tests rely on: on a graph small enough for
the oracle to run the whole layer, the oracle's outputs on an induced sub-problem equal, for the nodes the sub-problem
was built for, the oracle's outputs on the whole graph."""
import numpy as np

import oracle
import sampled_checks as sc
from circuit_synth import make_graph, make_tensors


def _case(k=8, D=32):
    g = make_graph("medium", seed=3, Nc=3000, Nn=2000, grid=(60, 50), evil=0.002)
    T = make_tensors(g.Nc, g.Nn, D, seed=3)
    rel = dict(near=oracle.relation(g.near, oracle.NORM_MEAN), pins=oracle.relation(g.pins, oracle.NORM_MEAN),
               pinned=oracle.relation(g.pinned, oracle.NORM_SYM))
    tr = {n: oracle.csr_transpose(rel[n].M, rel[n].N, rel[n].rowptr, rel[n].colidx, rel[n].vals) for n in rel}
    of = oracle.heteroconv_fwd(rel["near"], rel["pins"], rel["pinned"], T.X_cell, T.X_net, T.W, k, k)
    ob = oracle.heteroconv_bwd(rel["near"], rel["pins"], rel["pinned"], T.W, of, T.dY_cell, T.dY_net)
    return dict(g=g, T=T, D=D, k=k, rel=rel, tr=tr), of, ob


def test_forward_of_the_chosen_nodes_equals_the_whole_graph():
    r, of, _ = _case()
    g, T, k = r["g"], r["T"], r["k"]
    rng = np.random.default_rng(1)
    cells = np.sort(rng.choice(g.Nc, 40, replace=False))
    nets = np.unique(np.concatenate([rng.choice(g.Nn, 30, replace=False), [int(np.argmax(np.diff(r["rel"]["pins"].rowptr)))]]))
    sp = sc.induced_problem(r, cells, nets)
    assert len(sp["C"]) < g.Nc and len(sp["N"]) < g.Nn
    sub = oracle.heteroconv_fwd(sp["near"], sp["pins"], sp["pinned"], T.X_cell[sp["C"]], T.X_net[sp["N"]], T.W, k, k)
    lc, ln = sp["loc_cell"](cells), sp["loc_net"](nets)
    for nm in ("Y_cell", "H_near", "H_pinned", "Z_near", "Z_pinned", "mask", "l1_cell", "idx_cell", "vals_cell"):
        assert np.array_equal(sub[nm][lc], of[nm][cells]), nm
    for nm in ("Y_net", "H_pins", "l1_net", "idx_net"):
        assert np.array_equal(sub[nm][ln], of[nm][nets]), nm


def test_backward_of_the_chosen_sources_equals_the_whole_graph():
    r, of, ob = _case()
    g, T, k, tr = r["g"], r["T"], r["k"], r["tr"]
    rng = np.random.default_rng(2)
    src_c = np.sort(rng.choice(g.Nc, 25, replace=False))
    src_n = np.unique(np.concatenate([rng.choice(g.Nn, 15, replace=False), [int(np.argmax(np.diff(tr["pinned"][0])))]]))
    need = np.unique(np.concatenate([src_c, sc._rows_cols(tr["near"][0], tr["near"][1], src_c),
                                     sc._rows_cols(tr["pinned"][0], tr["pinned"][1], src_n)]))
    sp = sc.induced_problem(r, need, [], src_c, src_n)
    sub_f = oracle.heteroconv_fwd(sp["near"], sp["pins"], sp["pinned"], T.X_cell[sp["C"]], T.X_net[sp["N"]], T.W, k, k)
    assert np.array_equal(sub_f["mask"][sp["loc_cell"](need)], of["mask"][need])
    sub_b = oracle.heteroconv_bwd(sp["near"], sp["pins"], sp["pinned"], T.W, sub_f, T.dY_cell[sp["C"]], T.dY_net[sp["N"]])
    lc, ln = sp["loc_cell"](src_c), sp["loc_net"](src_n)
    # sums run over the same terms in the same order, so the values agree to the last bit
    assert np.array_equal(sub_b["dXs_cell"][lc], ob["dXs_cell"][src_c])
    assert np.array_equal(sub_b["l1_dxs_cell"][lc], ob["l1_dxs_cell"][src_c])
    assert np.array_equal(sub_b["dXs_net"][ln], ob["dXs_net"][src_n])
    assert np.array_equal(sub_b["dX_cell"][lc], ob["dX_cell"][src_c])
    # a sub-problem that lacks the destinations' forward does NOT reproduce the gradient (the check has teeth)
    bad = sc.induced_problem(r, src_c, [], src_c, src_n)
    bad_f = oracle.heteroconv_fwd(bad["near"], bad["pins"], bad["pinned"], T.X_cell[bad["C"]], T.X_net[bad["N"]], T.W, k, k)
    bad_b = oracle.heteroconv_bwd(bad["near"], bad["pins"], bad["pinned"], T.W, bad_f, T.dY_cell[bad["C"]], T.dY_net[bad["N"]])
    assert not np.array_equal(bad_b["dXs_cell"][bad["loc_cell"](src_c)], ob["dXs_cell"][src_c])
