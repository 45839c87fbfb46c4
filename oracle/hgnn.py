"""Oracle of the multi-layer training step (paper Section 4.1: stacked HeteroConv layers, ReLU between
layers, a per-cell regression read-out, MSE loss, Adam with weight decay), in fp64 numpy on top of the
single-layer oracle.

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and by nothing in the GPU package).

Model, for a batch of independent sub-graphs g that share the parameters:
    X^(0) = input features;  for l = 1..L:  (Y_cell, Y_net) = HeteroConv_l(X_cell^(l-1), X_net^(l-1)),
    X^(l) = ReLU(Y) for l < L,  X^(L) = Y;
    pred_i = X_cell^(L)[i, :] . w_head;   loss = mean over ALL cells of the batch of (pred_i - target_i)^2.
Parameters theta = [layer 1: self_near, neigh_near, self_pins, neigh_pins, pinned | layer 2 ... | w_head],
every layer weight [D, D] row-major.
Adam (Kingma & Ba) with the L2 form of weight decay (the gradient gets wd * theta added), bias-corrected.

Every function takes optional per-layer overrides so that a caller can "teacher-force" a layer with the
inputs / selections another implementation actually used; that keeps a comparison meaningful where fp32
rounding could flip a discrete decision (top-k, max-merge, ReLU sign) of a later layer.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np

from . import WEIGHT_NAMES, heteroconv_bwd, heteroconv_fwd
from . import per_relation as _pr


def _layer_fwd(rel, xc, xn, W, k):
    """k: one int for both node types, or per_relation.Ks (one K per edge type, paper Section 4.3)."""
    if isinstance(k, _pr.Ks):
        return _pr.heteroconv_fwd(*rel, xc, xn, W, k)
    return heteroconv_fwd(*rel, xc, xn, W, k, k)


def _layer_bwd(rel, W, saved, dYc, dYn):
    if "idx_cell_near" in saved:
        return _pr.heteroconv_bwd(*rel, W, saved, dYc, dYn)
    return heteroconv_bwd(*rel, W, saved, dYc, dYn)


def n_params(L: int, D: int) -> int:
    return L * 5 * D * D + D


def unpack(theta, L: int, D: int):
    """theta -> ([{name: [D,D]} per layer], w_head[D]) as fp64 views/copies."""
    theta = np.asarray(theta, dtype=np.float64)
    assert theta.shape == (n_params(L, D),)
    Ws = []
    for l in range(L):
        base = l * 5 * D * D
        Ws.append({n: theta[base + i * D * D: base + (i + 1) * D * D].reshape(D, D) for i, n in enumerate(WEIGHT_NAMES)})
    return Ws, theta[L * 5 * D * D:]


def pack(Ws: Sequence[Dict[str, np.ndarray]], w_head) -> np.ndarray:
    parts = [np.asarray(W[n], dtype=np.float64).ravel() for W in Ws for n in WEIGHT_NAMES]
    parts.append(np.asarray(w_head, dtype=np.float64).ravel())
    return np.concatenate(parts)


def forward_graph(rel, X_cell, X_net, Ws, w_head, k: int, layer_inputs: Optional[List] = None):
    """One sub-graph.  rel = (near, pins, pinned) oracle relations; k an int or per_relation.Ks.  layer_inputs[l] = (X_cell, X_net) overrides
    the input of layer l (l >= 1).  Returns dict(layers=[layer oracle outputs + inputs], pred)."""
    L = len(Ws)
    xc, xn = np.asarray(X_cell, dtype=np.float64), np.asarray(X_net, dtype=np.float64)
    layers = []
    for l in range(L):
        if layer_inputs is not None and l >= 1 and layer_inputs[l] is not None:
            xc, xn = (np.asarray(a, dtype=np.float64) for a in layer_inputs[l])
        o = _layer_fwd(rel, xc, xn, Ws[l], k)
        o["X_cell"], o["X_net"] = xc, xn
        layers.append(o)
        if l < L - 1:
            xc, xn = np.maximum(o["Y_cell"], 0.0), np.maximum(o["Y_net"], 0.0)
        else:
            xc, xn = o["Y_cell"], o["Y_net"]
    pred = xc @ np.asarray(w_head, dtype=np.float64)
    return dict(layers=layers, out_cell=xc, out_net=xn, pred=pred)


def loss_of(preds: Sequence[np.ndarray], targets: Sequence[np.ndarray]) -> float:
    n = sum(len(p) for p in preds)
    return float(sum(np.sum((p - np.asarray(t, dtype=np.float64)) ** 2) for p, t in zip(preds, targets)) / n)


def backward_graph(rel, fwd, Ws, w_head, target, n_total: int, saved_override: Optional[List] = None,
                   grad_override: Optional[List] = None):
    """Gradient of the batch loss with respect to this sub-graph's share.  saved_override[l] replaces the saved
    state (vals/idx/H/mask) of layer l; grad_override[l] = (dY_cell, dY_net) replaces the gradient arriving at the
    OUTPUT of layer l.  Returns dict(dW=[per layer {name: [D,D]}], dw_head, dpred, dY=[(dYc, dYn) per layer],
    dX=[(dXc, dXn) per layer])."""
    L = len(Ws)
    w_head = np.asarray(w_head, dtype=np.float64)
    dpred = 2.0 * (fwd["pred"] - np.asarray(target, dtype=np.float64)) / n_total
    dw_head = fwd["out_cell"].T @ dpred
    dYc = np.outer(dpred, w_head)
    dYn = np.zeros_like(fwd["out_net"])
    dW = [None] * L
    dYs, dXs = [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        if grad_override is not None and grad_override[l] is not None:
            dYc, dYn = (np.asarray(a, dtype=np.float64) for a in grad_override[l])
        lay = fwd["layers"][l]
        saved = lay if saved_override is None or saved_override[l] is None else saved_override[l]
        ob = _layer_bwd(rel, Ws[l], saved, dYc, dYn)
        dW[l] = ob["dW"]
        dYs[l] = (dYc, dYn)
        dXs[l] = (ob["dX_cell"], ob["dX_net"])
        if l >= 1:
            # ReLU between layer l-1 and l: its input was Y of layer l-1, its output X of layer l
            dYc = np.where(lay["X_cell"] > 0.0, ob["dX_cell"], 0.0)
            dYn = np.where(lay["X_net"] > 0.0, ob["dX_net"], 0.0)
    return dict(dW=dW, dw_head=dw_head, dpred=dpred, dY=dYs, dX=dXs)


def adam_step(theta, grad, m, v, lr: float, beta1: float, beta2: float, eps: float, weight_decay: float, t: int):
    """One Adam update (t = 1 for the first).  Returns (theta', m', v')."""
    theta, grad, m, v = (np.asarray(a, dtype=np.float64) for a in (theta, grad, m, v))
    g = grad + weight_decay * theta
    m2 = beta1 * m + (1.0 - beta1) * g
    v2 = beta2 * v + (1.0 - beta2) * g * g
    mhat = m2 / (1.0 - beta1 ** t)
    vhat = v2 / (1.0 - beta2 ** t)
    return theta - lr * mhat / (np.sqrt(vhat) + eps), m2, v2


def train_step(rels, X_cells, X_nets, targets, theta, m, v, L: int, D: int, k: int, lr=2e-4, beta1=0.9, beta2=0.999,
               eps=1e-8, weight_decay=1e-5, t=1):
    """Whole step on a batch of sub-graphs; k is one K for all or a list with one entry (int or per_relation.Ks) per
    sub-graph.  Returns dict(loss, grad, theta, m, v, fwd=[...], bwd=[...])."""
    Ws, w_head = unpack(theta, L, D)
    ks = list(k) if isinstance(k, (list, tuple)) and not isinstance(k, _pr.Ks) else [k] * len(rels)
    fwds = [forward_graph(r, xc, xn, Ws, w_head, kq) for r, xc, xn, kq in zip(rels, X_cells, X_nets, ks)]
    n_total = sum(len(f["pred"]) for f in fwds)
    loss = loss_of([f["pred"] for f in fwds], targets)
    bwds = [backward_graph(r, f, Ws, w_head, tg, n_total) for r, f, tg in zip(rels, fwds, targets)]
    gW = [{n: sum(b["dW"][l][n] for b in bwds) for n in WEIGHT_NAMES} for l in range(L)]
    grad = pack(gW, sum(b["dw_head"] for b in bwds))
    th2, m2, v2 = adam_step(theta, grad, m, v, lr, beta1, beta2, eps, weight_decay, t)
    return dict(loss=loss, grad=grad, theta=th2, m=m2, v=v2, fwd=fwds, bwd=bwds)
