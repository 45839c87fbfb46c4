"""Pins of the training-step oracle (oracle/hgnn.py) against things other than itself: central differences
of the loss in fp64, torch's Adam, and the single-layer oracle written out by hand."""
import numpy as np
import pytest
import torch

import oracle
from oracle import hgnn
from circuit_synth import make_graph


def _graph(seed, Nc=40, Nn=24, grid=(8, 5)):
    g = make_graph("tiny", seed=seed, Nc=Nc, Nn=Nn, grid=grid)
    rel = (oracle.relation(g.near, oracle.NORM_MEAN), oracle.relation(g.pins, oracle.NORM_MEAN),
           oracle.relation(g.pinned, oracle.NORM_SYM))
    return g, rel


def _batch(D, seeds=(3, 4)):
    rng = np.random.default_rng(11)
    rels, Xc, Xn, tg = [], [], [], []
    for s in seeds:
        g, rel = _graph(s)
        rels.append(rel)
        Xc.append(rng.standard_normal((g.Nc, D)))
        Xn.append(rng.standard_normal((g.Nn, D)))
        tg.append(rng.standard_normal(g.Nc))
    return rels, Xc, Xn, tg


def _loss(theta, rels, Xc, Xn, tg, L, D, k):
    Ws, wh = hgnn.unpack(theta, L, D)
    preds = [hgnn.forward_graph(r, a, b, Ws, wh, k)["pred"] for r, a, b in zip(rels, Xc, Xn)]
    return hgnn.loss_of(preds, tg)


@pytest.mark.parametrize("L", [1, 2, 3])
def test_gradient_matches_central_differences(L):
    D, k = 8, 3
    rels, Xc, Xn, tg = _batch(D)
    rng = np.random.default_rng(5 + L)
    theta = rng.uniform(-0.6, 0.6, hgnn.n_params(L, D))
    out = hgnn.train_step(rels, Xc, Xn, tg, theta, np.zeros_like(theta), np.zeros_like(theta), L, D, k)
    assert abs(out["loss"] - _loss(theta, rels, Xc, Xn, tg, L, D, k)) < 1e-14
    h = 1e-6
    for trial in range(6):
        d = rng.standard_normal(theta.shape)
        if trial >= 3:                                   # single-block directions: one weight matrix (or the head) at a time
            blk = rng.integers(0, L * 5 + 1)
            keep = np.zeros_like(d)
            lo = blk * D * D
            hi = lo + (D * D if blk < L * 5 else D)
            keep[lo:hi] = d[lo:hi]
            d = keep
        d /= np.linalg.norm(d)
        fd = (_loss(theta + h * d, rels, Xc, Xn, tg, L, D, k) - _loss(theta - h * d, rels, Xc, Xn, tg, L, D, k)) / (2 * h)
        an = float(out["grad"] @ d)
        assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (L, trial, fd, an)


def test_single_layer_model_is_the_layer_oracle_plus_readout():
    D, k, L = 8, 3, 1
    rels, Xc, Xn, tg = _batch(D, seeds=(7,))
    rng = np.random.default_rng(2)
    theta = rng.uniform(-0.5, 0.5, hgnn.n_params(L, D))
    Ws, wh = hgnn.unpack(theta, L, D)
    lay = oracle.heteroconv_fwd(*rels[0], Xc[0], Xn[0], Ws[0], k, k)
    pred = lay["Y_cell"] @ wh                               # no ReLU after the last layer
    out = hgnn.train_step(rels, Xc, Xn, tg, theta, np.zeros_like(theta), np.zeros_like(theta), L, D, k)
    assert np.allclose(out["fwd"][0]["pred"], pred, rtol=0, atol=1e-14)
    assert abs(out["loss"] - np.mean((pred - tg[0]) ** 2)) < 1e-14
    # the gradient arriving at the layer is the outer product of the read-out gradient and w_head
    dpred = 2 * (pred - tg[0]) / len(pred)
    ob = oracle.heteroconv_bwd(*rels[0], Ws[0], lay, np.outer(dpred, wh), np.zeros((Xn[0].shape[0], D)))
    for i, n in enumerate(oracle.WEIGHT_NAMES):
        assert np.allclose(out["grad"][i * D * D:(i + 1) * D * D].reshape(D, D), ob["dW"][n], rtol=0, atol=1e-14)
    assert np.allclose(out["grad"][5 * D * D:], lay["Y_cell"].T @ dpred, rtol=0, atol=1e-14)


def test_relu_sits_between_layers_only():
    D, k, L = 8, 3, 2
    rels, Xc, Xn, tg = _batch(D, seeds=(9,))
    rng = np.random.default_rng(3)
    Ws, wh = hgnn.unpack(rng.uniform(-0.5, 0.5, hgnn.n_params(L, D)), L, D)
    f = hgnn.forward_graph(rels[0], Xc[0], Xn[0], Ws, wh, k)
    assert np.array_equal(f["layers"][1]["X_cell"], np.maximum(f["layers"][0]["Y_cell"], 0))
    assert np.array_equal(f["layers"][1]["X_net"], np.maximum(f["layers"][0]["Y_net"], 0))
    assert (f["out_cell"] < 0).any()                        # the last layer's output is not clamped
    assert np.array_equal(f["out_cell"], f["layers"][1]["Y_cell"])


def test_batch_loss_is_the_mean_over_all_cells():
    D, k, L = 8, 3, 2
    rels, Xc, Xn, tg = _batch(D, seeds=(3, 4, 5))
    theta = np.random.default_rng(1).uniform(-0.5, 0.5, hgnn.n_params(L, D))
    z = np.zeros_like(theta)
    whole = hgnn.train_step(rels, Xc, Xn, tg, theta, z, z, L, D, k)
    parts = [hgnn.train_step(rels[i:i + 1], Xc[i:i + 1], Xn[i:i + 1], tg[i:i + 1], theta, z, z, L, D, k) for i in range(3)]
    n = np.array([len(t) for t in tg], dtype=np.float64)
    assert abs(whole["loss"] - sum(p["loss"] * w for p, w in zip(parts, n / n.sum()))) < 1e-14
    assert np.allclose(whole["grad"], sum(p["grad"] * w for p, w in zip(parts, n / n.sum())), rtol=0, atol=1e-14)


def test_adam_matches_torch():
    rng = np.random.default_rng(0)
    n = 257
    theta0 = rng.standard_normal(n)
    grads = [rng.standard_normal(n) * s for s in (1.0, 1e-3, 10.0, 1e-6)]
    lr, b1, b2, eps, wd = 2e-4, 0.9, 0.999, 1e-8, 1e-5
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    th, m, v = theta0.copy(), np.zeros(n), np.zeros(n)
    for t, g in enumerate(grads, start=1):
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, m, v = hgnn.adam_step(th, g, m, v, lr, b1, b2, eps, wd, t)
        assert np.allclose(th, p.detach().numpy(), rtol=1e-12, atol=1e-15), t


def test_gradient_with_one_k_per_edge_type_and_per_subgraph():
    """Sub-graphs that keep their own (k_near, k_pins, k_pinned): the batch gradient against central differences."""
    from oracle.per_relation import Ks
    D, L = 8, 2
    ks = [Ks.per_relation(2, 5, 3), 4]
    rels, Xc, Xn, tg = _batch(D)
    rng = np.random.default_rng(21)
    theta = rng.uniform(-0.6, 0.6, hgnn.n_params(L, D))

    def loss(th):
        Ws, wh = hgnn.unpack(th, L, D)
        preds = [hgnn.forward_graph(r, a, b, Ws, wh, k)["pred"] for r, a, b, k in zip(rels, Xc, Xn, ks)]
        return hgnn.loss_of(preds, tg)

    out = hgnn.train_step(rels, Xc, Xn, tg, theta, np.zeros_like(theta), np.zeros_like(theta), L, D, ks)
    assert abs(out["loss"] - loss(theta)) < 1e-14
    h = 1e-6
    for trial in range(5):
        d = rng.standard_normal(theta.shape)
        d /= np.linalg.norm(d)
        fd = (loss(theta + h * d) - loss(theta - h * d)) / (2 * h)
        an = float(out["grad"] @ d)
        assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (trial, fd, an)
