"""Oracle of the HeteroConv layer with one K per edge type (paper Section 4.3: graph-specific k_near,
k_pins and k_pinned, each profiled on its own sub-graph), in fp64 numpy on top of the single-step oracle.

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and by nothing in the GPU package).

Reading.  D-ReLU belongs to the module (edge type) that consumes the embedding, so every input of a module
is sparsified with that module's K:

    near   (cell->cell, SageConv mean):  Z_near   = f_{k_near}(X_cell) Wself_near + (A_near f_{k_near}(X_cell)) Wneigh_near
    pins   (cell->net,  SageConv mean):  Y_net    = f_{k_self}(X_net)  Wself_pins + (A_pins f_{k_pins}(X_cell)) Wneigh_pins
    pinned (net->cell,  GraphConv sym):  Z_pinned =                                (A_pinned f_{k_pinned}(X_net)) W_pinned
    Y_cell = max(Z_near, Z_pinned),  mask = [Z_near >= Z_pinned]

with k_self = k_pins for the per-edge-type setting; k_self is kept as its own argument so that the
per-node-type layer (k_near = k_pins = k_cell, k_self = k_pinned = k_net) is the same function.
The backward is the derivative of this forward with the selections and the mask held fixed: every use of an
embedding sends its gradient back through its own top-k positions, and the pieces add up densely.
"""
from __future__ import annotations

from typing import Dict, NamedTuple

import numpy as np

from . import WEIGHT_NAMES, Relation, csr_transpose, densify, spmm_bwd, spmm_fwd, topk


class Ks(NamedTuple):
    near: int     # cells, as source and self term of the near module
    pins: int     # cells, as source of the pins module
    self_: int    # nets, as self term of the pins module
    pinned: int   # nets, as source of the pinned module

    @staticmethod
    def per_relation(k_near: int, k_pins: int, k_pinned: int) -> "Ks":
        return Ks(k_near, k_pins, k_pins, k_pinned)

    @staticmethod
    def per_node_type(k_cell: int, k_net: int) -> "Ks":
        return Ks(k_cell, k_cell, k_net, k_net)


def _w(W) -> Dict[str, np.ndarray]:
    return {n: np.asarray(W[n], dtype=np.float64) for n in WEIGHT_NAMES}


def heteroconv_fwd(near: Relation, pins: Relation, pinned: Relation, X_cell, X_net, W, ks: Ks):
    X_cell, X_net = np.asarray(X_cell, dtype=np.float64), np.asarray(X_net, dtype=np.float64)
    D = X_cell.shape[1]
    W = _w(W)
    o = {}
    o["vals_cell_near"], o["idx_cell_near"] = topk(X_cell, ks.near)
    o["vals_cell_pins"], o["idx_cell_pins"] = topk(X_cell, ks.pins)
    o["vals_net_self"], o["idx_net_self"] = topk(X_net, ks.self_)
    o["vals_net_pinned"], o["idx_net_pinned"] = topk(X_net, ks.pinned)
    aW = {n: np.abs(W[n]) for n in WEIGHT_NAMES}

    def aggregate(rel, vals, idx):
        H, _, l1 = spmm_fwd(rel.rowptr, rel.colidx, rel.vals, vals, idx, D, want_l1elem=True)
        return H, l1

    # near
    Xs = densify(o["vals_cell_near"], o["idx_cell_near"], D)
    o["H_near"], habs = aggregate(near, o["vals_cell_near"], o["idx_cell_near"])
    o["Z_near"] = Xs @ W["self_near"] + o["H_near"] @ W["neigh_near"]
    l1_near = np.abs(Xs) @ aW["self_near"] + habs @ aW["neigh_near"]
    # pins
    Xs = densify(o["vals_net_self"], o["idx_net_self"], D)
    o["H_pins"], habs = aggregate(pins, o["vals_cell_pins"], o["idx_cell_pins"])
    o["Y_net"] = Xs @ W["self_pins"] + o["H_pins"] @ W["neigh_pins"]
    o["l1_net"] = np.abs(Xs) @ aW["self_pins"] + habs @ aW["neigh_pins"]
    # pinned
    o["H_pinned"], habs = aggregate(pinned, o["vals_net_pinned"], o["idx_net_pinned"])
    o["Z_pinned"] = o["H_pinned"] @ W["pinned"]
    l1_pinned = habs @ aW["pinned"]
    # merge at the cells: element-wise max, ties to the near branch
    o["mask"] = (o["Z_near"] >= o["Z_pinned"]).astype(np.uint8)
    o["Y_cell"] = np.where(o["mask"] == 1, o["Z_near"], o["Z_pinned"])
    o["l1_cell"] = np.maximum(l1_near, l1_pinned)
    return o


def _scatter(G, idx, D):
    """Dense [n, D] array holding G[j, t] at column idx[j, t] (columns of a row are distinct)."""
    out = np.zeros((G.shape[0], D))
    np.put_along_axis(out, np.asarray(idx, dtype=np.int64), G, axis=1)
    return out


def heteroconv_bwd(near: Relation, pins: Relation, pinned: Relation, W, saved, dY_cell, dY_net):
    """``saved``: the four index sets (idx_cell_near, idx_cell_pins, idx_net_self, idx_net_pinned), the values of the
    two self-term sets (vals_cell_near, vals_net_self), H_near, H_pins, H_pinned and mask.  Returns dX_cell, dX_net,
    dW and, per element of dX, the sum of the absolute values of the terms that were added up (l1_dX_*)."""
    dY_cell, dY_net = np.asarray(dY_cell, dtype=np.float64), np.asarray(dY_net, dtype=np.float64)
    D = dY_cell.shape[1]
    W = _w(W)
    mask = np.asarray(saved["mask"]) == 1
    dZ_near = np.where(mask, dY_cell, 0.0)
    dZ_pinned = np.where(mask, 0.0, dY_cell)
    H = {n: np.asarray(saved["H_" + n], dtype=np.float64) for n in ("near", "pins", "pinned")}

    dW = {}
    Xs = densify(saved["vals_cell_near"], saved["idx_cell_near"], D)
    dW["self_near"] = Xs.T @ dZ_near
    dW["neigh_near"] = H["near"].T @ dZ_near
    Xs = densify(saved["vals_net_self"], saved["idx_net_self"], D)
    dW["self_pins"] = Xs.T @ dY_net
    dW["neigh_pins"] = H["pins"].T @ dY_net
    dW["pinned"] = H["pinned"].T @ dZ_pinned

    def gather(rel, dZ, Wn, idx):
        """Transposed SpMM of dH = dZ Wn^T, sampled at the source rows' saved columns, scattered to dense."""
        t_rowptr, t_colidx, t_vals = csr_transpose(rel.M, rel.N, rel.rowptr, rel.colidx, rel.vals)
        G, _, l1 = spmm_bwd(t_rowptr, t_colidx, t_vals, dZ @ W[Wn].T, idx, want_l1elem=True)
        return _scatter(G, idx, D), _scatter(l1, idx, D)

    def sample(dZ, Wn, idx):
        """Self term dZ Wn^T kept at the saved columns only."""
        S = dZ @ W[Wn].T
        G = np.take_along_axis(S, np.asarray(idx, dtype=np.int64), axis=1)
        return _scatter(G, idx, D), _scatter(np.abs(G), idx, D)

    pieces_cell = [gather(near, dZ_near, "neigh_near", saved["idx_cell_near"]),
                   sample(dZ_near, "self_near", saved["idx_cell_near"]),
                   gather(pins, dY_net, "neigh_pins", saved["idx_cell_pins"])]
    pieces_net = [gather(pinned, dZ_pinned, "pinned", saved["idx_net_pinned"]),
                  sample(dY_net, "self_pins", saved["idx_net_self"])]
    return dict(
        dX_cell=sum(p[0] for p in pieces_cell), l1_dX_cell=sum(p[1] for p in pieces_cell),
        dX_net=sum(p[0] for p in pieces_net), l1_dX_net=sum(p[1] for p in pieces_net), dW=dW)
