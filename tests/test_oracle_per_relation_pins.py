"""Pins of the per-edge-type-K layer oracle (oracle/per_relation.py) against things other than itself:
central differences of a scalar functional in fp64, the dense SageConv / GraphConv formulas evaluated with scipy
when no entry is dropped, the independently pinned single-K layer oracle where the K coincide, and the
nesting of top-k sets."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from oracle import per_relation as pr
from circuit_synth import make_graph


def _setup(seed=2, Nc=48, Nn=30, grid=(8, 6), D=12):
    g = make_graph("tiny", seed=seed, Nc=Nc, Nn=Nn, grid=grid)
    rel = (oracle.relation(g.near, oracle.NORM_MEAN), oracle.relation(g.pins, oracle.NORM_MEAN),
           oracle.relation(g.pinned, oracle.NORM_SYM))
    rng = np.random.default_rng(100 + seed)
    Xc, Xn = rng.standard_normal((Nc, D)), rng.standard_normal((Nn, D))
    W = {n: rng.uniform(-0.5, 0.5, (D, D)) for n in oracle.WEIGHT_NAMES}
    Rc, Rn = rng.standard_normal((Nc, D)), rng.standard_normal((Nn, D))
    return g, rel, Xc, Xn, W, Rc, Rn


def _functional(rel, Xc, Xn, W, ks, Rc, Rn):
    o = pr.heteroconv_fwd(*rel, Xc, Xn, W, ks)
    return float(np.sum(o["Y_cell"] * Rc) + np.sum(o["Y_net"] * Rn))


@pytest.mark.parametrize("ks", [pr.Ks.per_relation(3, 7, 5), pr.Ks.per_relation(8, 2, 4), pr.Ks(5, 9, 2, 6)])
def test_backward_is_the_derivative_of_the_forward(ks):
    """L = <Y_cell, Rc> + <Y_net, Rn>: dL/dX and dL/dW from the backward against central differences.  The
    perturbations are far smaller than the gaps between the entries of a row, so no selection changes."""
    g, rel, Xc, Xn, W, Rc, Rn = _setup()
    fwd = pr.heteroconv_fwd(*rel, Xc, Xn, W, ks)
    bwd = pr.heteroconv_bwd(*rel, W, fwd, Rc, Rn)
    rng = np.random.default_rng(7)
    h = 1e-6
    for trial in range(4):
        dc, dn = rng.standard_normal(Xc.shape), rng.standard_normal(Xn.shape)
        fd = (_functional(rel, Xc + h * dc, Xn + h * dn, W, ks, Rc, Rn)
              - _functional(rel, Xc - h * dc, Xn - h * dn, W, ks, Rc, Rn)) / (2 * h)
        an = float(np.sum(bwd["dX_cell"] * dc) + np.sum(bwd["dX_net"] * dn))
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (trial, fd, an)
    for name in oracle.WEIGHT_NAMES:
        dw = rng.standard_normal(W[name].shape)
        Wp, Wm = dict(W), dict(W)
        Wp[name], Wm[name] = W[name] + h * dw, W[name] - h * dw
        fd = (_functional(rel, Xc, Xn, Wp, ks, Rc, Rn) - _functional(rel, Xc, Xn, Wm, ks, Rc, Rn)) / (2 * h)
        an = float(np.sum(bwd["dW"][name] * dw))
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, fd, an)


def test_single_entry_perturbations_see_every_use_of_an_embedding():
    """A cell entry inside the k_pins set but outside the k_near set feeds only the pins module; one inside
    both feeds near (source and self term) and pins.  Central differences entry by entry."""
    ks = pr.Ks.per_relation(3, 7, 5)
    g, rel, Xc, Xn, W, Rc, Rn = _setup(seed=4)
    fwd = pr.heteroconv_fwd(*rel, Xc, Xn, W, ks)
    bwd = pr.heteroconv_bwd(*rel, W, fwd, Rc, Rn)
    h = 1e-6
    for j in (0, 5, 17):
        for c in range(Xc.shape[1]):
            E = np.zeros_like(Xc)
            E[j, c] = h
            fd = (_functional(rel, Xc + E, Xn, W, ks, Rc, Rn) - _functional(rel, Xc - E, Xn, W, ks, Rc, Rn)) / (2 * h)
            assert abs(fd - bwd["dX_cell"][j, c]) <= 1e-6 * max(1.0, abs(fd)), (j, c)
            if c not in fwd["idx_cell_pins"][j]:
                assert bwd["dX_cell"][j, c] == 0.0
    for j in (1, 9):
        for c in range(Xn.shape[1]):
            E = np.zeros_like(Xn)
            E[j, c] = h
            fd = (_functional(rel, Xc, Xn + E, W, ks, Rc, Rn) - _functional(rel, Xc, Xn - E, W, ks, Rc, Rn)) / (2 * h)
            assert abs(fd - bwd["dX_net"][j, c]) <= 1e-6 * max(1.0, abs(fd)), (j, c)


def _dense(rel):
    return sp.csr_matrix((rel.vals.astype(np.float64), rel.colidx, rel.rowptr), shape=(rel.M, rel.N))


def test_k_equal_D_is_the_plain_sageconv_graphconv_layer():
    """With k = D nothing is dropped: the layer is SageConv(mean) / GraphConv(sym) on the raw embeddings, and its
    backward the textbook one (scipy sparse products, written from the module definitions)."""
    g, rel, Xc, Xn, W, Rc, Rn = _setup(seed=5)
    D = Xc.shape[1]
    ks = pr.Ks.per_relation(D, D, D)
    A_near, A_pins, A_pinned = (_dense(r) for r in rel)
    Zn = Xc @ W["self_near"] + (A_near @ Xc) @ W["neigh_near"]
    Yn = Xn @ W["self_pins"] + (A_pins @ Xc) @ W["neigh_pins"]
    Zp = (A_pinned @ Xn) @ W["pinned"]
    o = pr.heteroconv_fwd(*rel, Xc, Xn, W, ks)
    np.testing.assert_allclose(o["Y_cell"], np.maximum(Zn, Zp), rtol=0, atol=1e-12)
    np.testing.assert_allclose(o["Y_net"], Yn, rtol=0, atol=1e-12)
    b = pr.heteroconv_bwd(*rel, W, o, Rc, Rn)
    m = Zn >= Zp
    dZn, dZp = Rc * m, Rc * ~m
    dXc = dZn @ W["self_near"].T + A_near.T @ (dZn @ W["neigh_near"].T) + A_pins.T @ (Rn @ W["neigh_pins"].T)
    dXn = Rn @ W["self_pins"].T + A_pinned.T @ (dZp @ W["pinned"].T)
    np.testing.assert_allclose(b["dX_cell"], dXc, rtol=0, atol=1e-12)
    np.testing.assert_allclose(b["dX_net"], dXn, rtol=0, atol=1e-12)
    np.testing.assert_allclose(b["dW"]["neigh_pins"], (A_pins @ Xc).T @ Rn, rtol=0, atol=1e-12)
    np.testing.assert_allclose(b["dW"]["pinned"], (A_pinned @ Xn).T @ dZp, rtol=0, atol=1e-12)


@pytest.mark.parametrize("kc,kn", [(4, 4), (3, 6), (12, 1)])
def test_coinciding_k_reduce_to_the_single_k_layer_oracle(kc, kn):
    """Ks.per_node_type is the layer the C oracle computes (pinned on its own elsewhere)."""
    g, rel, Xc, Xn, W, Rc, Rn = _setup(seed=6)
    a = pr.heteroconv_fwd(*rel, Xc, Xn, W, pr.Ks.per_node_type(kc, kn))
    c = oracle.heteroconv_fwd(*rel, Xc, Xn, W, kc, kn)
    assert np.array_equal(a["idx_cell_near"], c["idx_cell"]) and np.array_equal(a["idx_cell_pins"], c["idx_cell"])
    assert np.array_equal(a["idx_net_self"], c["idx_net"]) and np.array_equal(a["idx_net_pinned"], c["idx_net"])
    for n in ("H_near", "H_pins", "H_pinned", "Y_cell", "Y_net", "l1_cell", "l1_net"):
        np.testing.assert_allclose(a[n], c[n], rtol=0, atol=1e-12, err_msg=n)
    assert np.array_equal(a["mask"], c["mask"])
    ab = pr.heteroconv_bwd(*rel, W, a, Rc, Rn)
    cb = oracle.heteroconv_bwd(*rel, W, c, Rc, Rn)
    np.testing.assert_allclose(ab["dX_cell"], cb["dX_cell"], rtol=0, atol=1e-12)
    np.testing.assert_allclose(ab["dX_net"], cb["dX_net"], rtol=0, atol=1e-12)
    for n in oracle.WEIGHT_NAMES:
        np.testing.assert_allclose(ab["dW"][n], cb["dW"][n], rtol=0, atol=1e-12, err_msg=n)


def test_topk_sets_are_nested_and_gradient_support_is_the_larger_set():
    ks = pr.Ks.per_relation(2, 6, 4)
    g, rel, Xc, Xn, W, Rc, Rn = _setup(seed=8)
    o = pr.heteroconv_fwd(*rel, Xc, Xn, W, ks)
    for small, large in (("idx_cell_near", "idx_cell_pins"), ("idx_net_pinned", "idx_net_self")):
        for r in range(o[small].shape[0]):
            assert set(o[small][r]) <= set(o[large][r])
    b = pr.heteroconv_bwd(*rel, W, o, Rc, Rn)
    support = np.zeros(Xc.shape, dtype=bool)
    np.put_along_axis(support, o["idx_cell_pins"].astype(np.int64), True, axis=1)
    assert not np.any(b["dX_cell"][~support])
    # rows with at least one outgoing pins edge carry gradient on every position of the larger set
    t_rowptr, _, _ = oracle.csr_transpose(rel[1].M, rel[1].N, rel[1].rowptr, rel[1].colidx, rel[1].vals)
    has_out = np.diff(t_rowptr) > 0
    assert np.all(b["dX_cell"][has_out][support[has_out]] != 0.0)
