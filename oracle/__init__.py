"""ctypes front-end of the CPU oracle (``dr_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg.  The GPU library never imports or calls it,
and nothing here imports the GPU package.

All floating-point inputs are widened to fp64 exactly before the C code sees
them; all floating-point results come back as fp64 arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dr_oracle.c")
_LIB = os.path.join(_HERE, "libdr_oracle.so")

NORM_MEAN = 0
NORM_SYM = 1

WEIGHT_NAMES = ("self_near", "neigh_near", "self_pins", "neigh_pins", "pinned")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


class _Csr(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("N", ctypes.c_int64),
                ("rowptr", ctypes.c_void_p), ("colidx", ctypes.c_void_p), ("vals", ctypes.c_void_p)]


class _Weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in WEIGHT_NAMES]


def _p(a: Optional[np.ndarray]):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.float32)


# ---------------------------------------------------------------------------
# single steps
# ---------------------------------------------------------------------------

def topk(X, k: int):
    """D-ReLU: returns (vals[n,k] fp64, idx[n,k] int32), survivors in ascending column order."""
    X = _f64(X)
    n, D = X.shape
    vals = np.empty((n, k), dtype=np.float64)
    idx = np.empty((n, k), dtype=np.int32)
    rc = _load().orc_topk(_p(X), ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int32(k), _p(vals), _p(idx))
    if rc != 0:
        raise ValueError("orc_topk: bad arguments or non-finite input")
    return vals, idx


def densify(vals, idx, D: int) -> np.ndarray:
    vals, idx = _f64(vals), _i32(idx)
    n, k = vals.shape
    out = np.empty((n, D), dtype=np.float64)
    _load().orc_densify(_p(vals), _p(idx), ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int32(k), _p(out))
    return out


def csr_normalize(mode: int, n_rows: int, n_cols: int, rowptr, colidx) -> np.ndarray:
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    vals = np.empty(colidx.shape[0], dtype=np.float32)
    rc = _load().orc_csr_normalize(ctypes.c_int(mode), ctypes.c_int64(n_rows), ctypes.c_int64(n_cols),
                                   _p(rowptr), _p(colidx), _p(vals))
    if rc != 0:
        raise ValueError("orc_csr_normalize: bad mode")
    return vals


def spmm_fwd(rowptr, colidx, avals, xs_vals, xs_idx, D: int, want_l1elem: bool = False):
    """H = A f(X).  Returns (H[M,D], l1row[M]) or (H, l1row, l1elem[M,D])."""
    rowptr, colidx, avals = _i32(rowptr), _i32(colidx), _f32(avals)
    xs_vals, xs_idx = _f64(xs_vals), _i32(xs_idx)
    M = rowptr.shape[0] - 1
    k = xs_vals.shape[1]
    H = np.empty((M, D), dtype=np.float64)
    l1row = np.empty(M, dtype=np.float64)
    l1elem = np.empty((M, D), dtype=np.float64) if want_l1elem else None
    _load().orc_spmm_fwd(ctypes.c_int64(M), _p(rowptr), _p(colidx), _p(avals), _p(xs_vals), _p(xs_idx),
                         ctypes.c_int32(D), ctypes.c_int32(k), _p(H), _p(l1elem), _p(l1row))
    return (H, l1row, l1elem) if want_l1elem else (H, l1row)


def csr_transpose(n_rows: int, n_cols: int, rowptr, colidx, vals=None):
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    vals = None if vals is None else _f32(vals)
    t_rowptr = np.empty(n_cols + 1, dtype=np.int32)
    t_colidx = np.empty(colidx.shape[0], dtype=np.int32)
    t_vals = None if vals is None else np.empty(colidx.shape[0], dtype=np.float32)
    _load().orc_csr_transpose(ctypes.c_int64(n_rows), ctypes.c_int64(n_cols), _p(rowptr), _p(colidx), _p(vals),
                              _p(t_rowptr), _p(t_colidx), _p(t_vals))
    return t_rowptr, t_colidx, t_vals


def spmm_bwd(t_rowptr, t_colidx, t_vals, dH, xs_idx, want_l1elem: bool = False):
    """G[j,t] = sum_e At[j,e] dH[col_e, idx[j,t]].  Returns (G[N,k], l1row[N]) (+ l1elem[N,k])."""
    t_rowptr, t_colidx, t_vals = _i32(t_rowptr), _i32(t_colidx), _f32(t_vals)
    dH, xs_idx = _f64(dH), _i32(xs_idx)
    N = t_rowptr.shape[0] - 1
    D = dH.shape[1]
    k = xs_idx.shape[1]
    G = np.empty((N, k), dtype=np.float64)
    l1row = np.empty(N, dtype=np.float64)
    l1elem = np.empty((N, k), dtype=np.float64) if want_l1elem else None
    _load().orc_spmm_bwd(ctypes.c_int64(N), _p(t_rowptr), _p(t_colidx), _p(t_vals), _p(dH), ctypes.c_int32(D),
                         _p(xs_idx), ctypes.c_int32(k), _p(G), _p(l1elem), _p(l1row))
    return (G, l1row, l1elem) if want_l1elem else (G, l1row)


# ---------------------------------------------------------------------------
# the layer
# ---------------------------------------------------------------------------

@dataclass
class Relation:
    """CSR of one relation: M destination rows, N source columns, fp32 edge values."""
    M: int
    N: int
    rowptr: np.ndarray
    colidx: np.ndarray
    vals: np.ndarray

    def _c(self) -> _Csr:
        self.rowptr, self.colidx, self.vals = _i32(self.rowptr), _i32(self.colidx), _f32(self.vals)
        return _Csr(self.M, self.N, self.rowptr.ctypes.data, self.colidx.ctypes.data, self.vals.ctypes.data)


def relation(pattern, mode: int) -> Relation:
    """Attach the module's edge values to a sparsity pattern (anything with n_rows, n_cols, rowptr, colidx)."""
    vals = csr_normalize(mode, pattern.n_rows, pattern.n_cols, pattern.rowptr, pattern.colidx)
    return Relation(pattern.n_rows, pattern.n_cols, _i32(pattern.rowptr), _i32(pattern.colidx), vals)


def _weights(W: Dict[str, np.ndarray]):
    keep = {n: _f64(W[n]) for n in WEIGHT_NAMES}
    return keep, _Weights(*[keep[n].ctypes.data for n in WEIGHT_NAMES])


def heteroconv_fwd(near: Relation, pins: Relation, pinned: Relation, X_cell, X_net, W, k_cell: int, k_net: int):
    X_cell, X_net = _f64(X_cell), _f64(X_net)
    Nc, D = X_cell.shape
    Nn = X_net.shape[0]
    keep, cw = _weights(W)
    o = dict(
        vals_cell=np.empty((Nc, k_cell)), idx_cell=np.empty((Nc, k_cell), dtype=np.int32),
        vals_net=np.empty((Nn, k_net)), idx_net=np.empty((Nn, k_net), dtype=np.int32),
        H_near=np.empty((Nc, D)), H_pins=np.empty((Nn, D)), H_pinned=np.empty((Nc, D)),
        Z_near=np.empty((Nc, D)), Z_pinned=np.empty((Nc, D)),
        Y_cell=np.empty((Nc, D)), Y_net=np.empty((Nn, D)), mask=np.empty((Nc, D), dtype=np.uint8),
        l1_cell=np.empty((Nc, D)), l1_net=np.empty((Nn, D)),
    )
    cn, cp, cq = near._c(), pins._c(), pinned._c()
    rc = _load().orc_heteroconv_fwd(
        ctypes.c_int64(Nc), ctypes.c_int64(Nn), ctypes.c_int32(D), ctypes.c_int32(k_cell), ctypes.c_int32(k_net),
        ctypes.byref(cn), ctypes.byref(cp), ctypes.byref(cq), _p(X_cell), _p(X_net), ctypes.byref(cw),
        _p(o["vals_cell"]), _p(o["idx_cell"]), _p(o["vals_net"]), _p(o["idx_net"]),
        _p(o["H_near"]), _p(o["H_pins"]), _p(o["H_pinned"]), _p(o["Z_near"]), _p(o["Z_pinned"]),
        _p(o["Y_cell"]), _p(o["Y_net"]), _p(o["mask"]), _p(o["l1_cell"]), _p(o["l1_net"]))
    if rc != 0:
        raise ValueError("orc_heteroconv_fwd: inconsistent shapes or non-finite input")
    return o


def heteroconv_bwd(near: Relation, pins: Relation, pinned: Relation, W, saved, dY_cell, dY_net):
    """``saved`` needs vals_cell, idx_cell, vals_net, idx_net, H_near, H_pins, H_pinned, mask."""
    dY_cell, dY_net = _f64(dY_cell), _f64(dY_net)
    Nc, D = dY_cell.shape
    Nn = dY_net.shape[0]
    vc, ic = _f64(saved["vals_cell"]), _i32(saved["idx_cell"])
    vn, inn = _f64(saved["vals_net"]), _i32(saved["idx_net"])
    Hn, Hp, Hq = _f64(saved["H_near"]), _f64(saved["H_pins"]), _f64(saved["H_pinned"])
    mask = np.ascontiguousarray(saved["mask"], dtype=np.uint8)
    kc, kn = vc.shape[1], vn.shape[1]
    keep, cw = _weights(W)
    o = dict(
        dX_cell=np.empty((Nc, D)), dX_net=np.empty((Nn, D)),
        dXs_cell=np.empty((Nc, kc)), dXs_net=np.empty((Nn, kn)),
        dW={n: np.empty((D, D)) for n in WEIGHT_NAMES},
        l1_dxs_cell=np.empty((Nc, kc)), l1_dxs_net=np.empty((Nn, kn)),
    )
    cn, cp, cq = near._c(), pins._c(), pinned._c()
    rc = _load().orc_heteroconv_bwd(
        ctypes.c_int64(Nc), ctypes.c_int64(Nn), ctypes.c_int32(D), ctypes.c_int32(kc), ctypes.c_int32(kn),
        ctypes.byref(cn), ctypes.byref(cp), ctypes.byref(cq), ctypes.byref(cw),
        _p(vc), _p(ic), _p(vn), _p(inn), _p(Hn), _p(Hp), _p(Hq), _p(mask), _p(dY_cell), _p(dY_net),
        _p(o["dX_cell"]), _p(o["dX_net"]), _p(o["dXs_cell"]), _p(o["dXs_net"]),
        *[_p(o["dW"][n]) for n in WEIGHT_NAMES],
        _p(o["l1_dxs_cell"]), _p(o["l1_dxs_net"]))
    if rc != 0:
        raise ValueError("orc_heteroconv_bwd failed")
    return o
