"""Thin ctypes binding of libdrcgnn.so: argument marshalling only.

Every function has the name of the C entry point it calls (see ``include/dr_circuitgnn.h``) and does
no arithmetic of its own.  Tensors are torch CUDA tensors used purely as device-memory handles
(``data_ptr()``); streams are taken from ``torch.cuda.current_stream()`` unless given.  A missing or
unloadable library raises: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Dict, Optional, Sequence

import torch

from . import build as _build

DR_OK = 0
DR_ERR_INVALID_ARG = -1
DR_ERR_UNSUPPORTED = -2
DR_ERR_HIP = -3
DR_ERR_WORKSPACE = -4
DR_NORM_MEAN = 0
DR_NORM_SYM = 1
DR_OVERLAP_AUTO = 0
DR_OVERLAP_ON = 1
DR_OVERLAP_OFF = 2

WEIGHT_NAMES = ("self_near", "neigh_near", "self_pins", "neigh_pins", "pinned")
EXPORTS = (
    "dr_last_error", "dr_abi_version", "dr_topk", "dr_spmm_fwd", "dr_spmm_bwd",
    "dr_spmm_plan_create", "dr_spmm_plan_info", "dr_spmm_bwd_planned", "dr_spmm_plan_destroy",
    "dr_topk_ranked", "dr_spmm_fwd_adaptive", "dr_degree_edge_classes", "dr_spmm_bwd_adaptive",
    "dr_csr_transpose_workspace_bytes", "dr_csr_transpose",
    "dr_csr_normalize_workspace_bytes", "dr_csr_normalize", "dr_csr_normalize_noalloc",
    "heteroconv_create", "heteroconv_create_per_relation", "heteroconv_get_k", "heteroconv_profile_k", "heteroconv_fwd", "heteroconv_bwd", "heteroconv_get_transpose", "heteroconv_destroy",
    "heteroconv_profile", "heteroconv_num_kernels", "heteroconv_kernel_name", "heteroconv_kernel_times",
    "heteroconv_set_overlap", "heteroconv_set_cell_order",
    "dr_pipeline_create", "dr_pipeline_submit", "dr_pipeline_acquire", "dr_pipeline_relations", "dr_pipeline_release",
    "dr_pipeline_destroy",
    "hgnn_num_params", "hgnn_create", "hgnn_create_batched", "hgnn_train_step", "hgnn_set_inspection", "hgnn_get_layer_buffers", "hgnn_destroy",
)


class DrError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libdrcgnn error {code}: {message}")
        self.code = code


class dr_csr(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int64), ("n_cols", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("rowptr", ctypes.c_void_p), ("colidx", ctypes.c_void_p), ("vals", ctypes.c_void_p)]


class dr_heteroconv_weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in WEIGHT_NAMES]


class dr_heteroconv_saved(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("vals_cell", "idx_cell", "vals_net", "idx_net", "H_near", "H_pins", "H_pinned", "mask",
                 "vals_cell_pins", "idx_cell_pins", "vals_net_self", "idx_net_self")]


_lib = None
_hip = None


def library_path() -> str:
    return _build.LIB


def hip_runtime() -> ctypes.CDLL:
    """The HIP runtime PyTorch itself uses.  libdrcgnn needs ``libamdhip64.so.7``; loading torch's copy
    first makes the dynamic loader resolve that soname to the same runtime, so streams and device
    pointers are shared between PyTorch and the library."""
    global _hip
    if _hip is None:
        bundled = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
        _hip = ctypes.CDLL(bundled if os.path.exists(bundled) else "libamdhip64.so", mode=ctypes.RTLD_GLOBAL)
    return _hip


def load() -> ctypes.CDLL:
    """Load the in-tree library (building it first only if no built library exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build(verbose=False)
        hip_runtime()
        lib = ctypes.CDLL(_build.LIB)
        lib.dr_last_error.restype = ctypes.c_char_p
        lib.dr_csr_transpose_workspace_bytes.restype = ctypes.c_size_t
        lib.dr_csr_normalize_workspace_bytes.restype = ctypes.c_size_t
        lib.heteroconv_kernel_name.restype = ctypes.c_char_p
        lib.hgnn_num_params.restype = ctypes.c_int64
        _lib = lib
    return _lib


def _check(rc: int) -> None:
    if rc != DR_OK:
        raise DrError(rc, load().dr_last_error().decode())


def _ptr(t):
    """Device address of a tensor; None -> NULL; a plain int is taken as an address (library-owned buffers)."""
    if t is None:
        return ctypes.c_void_p(0)
    return ctypes.c_void_p(t if isinstance(t, int) else t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


@dataclass
class Csr:
    """Device CSR of one relation (rows = destinations, columns = sources)."""
    n_rows: int
    n_cols: int
    rowptr: torch.Tensor            # int32 [n_rows+1]
    colidx: torch.Tensor            # int32 [nnz]
    vals: Optional[torch.Tensor]    # float32 [nnz] or None

    @property
    def nnz(self) -> int:
        return int(self.colidx.shape[0])

    def c(self) -> dr_csr:
        return dr_csr(self.n_rows, self.n_cols, self.nnz, self.rowptr.data_ptr(), self.colidx.data_ptr(),
                      0 if self.vals is None else self.vals.data_ptr())


def dr_last_error() -> str:
    return load().dr_last_error().decode()


def dr_abi_version() -> int:
    return int(load().dr_abi_version())


def dr_topk(X: torch.Tensor, k: int, vals: torch.Tensor, idx: torch.Tensor, stream=None) -> None:
    n, D = X.shape
    _check(load().dr_topk(_ptr(X), ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int32(k), _ptr(vals), _ptr(idx),
                          _stream(stream)))


def dr_spmm_fwd(A: Csr, xs_vals: torch.Tensor, xs_idx: torch.Tensor, D: int, k: int, H: torch.Tensor,
                stream=None) -> None:
    a = A.c()
    _check(load().dr_spmm_fwd(ctypes.byref(a), _ptr(xs_vals), _ptr(xs_idx), ctypes.c_int32(D), ctypes.c_int32(k),
                              _ptr(H), _stream(stream)))


def dr_spmm_bwd(At: Csr, dH: torch.Tensor, xs_idx: torch.Tensor, D: int, k: int, dXs: torch.Tensor,
                accumulate: bool = False, stream=None) -> None:
    a = At.c()
    _check(load().dr_spmm_bwd(ctypes.byref(a), _ptr(dH), _ptr(xs_idx), ctypes.c_int32(D), ctypes.c_int32(k),
                              _ptr(dXs), ctypes.c_int(1 if accumulate else 0), _stream(stream)))


class SpmmPlan:
    """Owner of a ``dr_spmm_plan*`` (dr_spmm_plan_create / dr_spmm_plan_destroy) for one transposed relation."""

    def __init__(self, At: Csr, D: int, row_order: Optional[torch.Tensor] = None, stream=None):
        self.D, self.n_rows = D, At.n_rows
        self._p = ctypes.c_void_p(0)
        a = At.c()
        _check(load().dr_spmm_plan_create(ctypes.byref(self._p), ctypes.byref(a), _ptr(row_order), ctypes.c_int32(D),
                                          _stream(stream)))

    def dr_spmm_plan_info(self):
        """(number of tiles, stored edges per distinct gathered row)."""
        n, r = ctypes.c_int64(0), ctypes.c_double(0.0)
        _check(load().dr_spmm_plan_info(self._p, ctypes.byref(n), ctypes.byref(r)))
        return int(n.value), float(r.value)

    def dr_spmm_bwd_planned(self, dH: torch.Tensor, xs_idx: torch.Tensor, k: int, dXs: torch.Tensor, accumulate: bool = False,
                            stream=None) -> None:
        _check(load().dr_spmm_bwd_planned(self._p, _ptr(dH), _ptr(xs_idx), ctypes.c_int32(k), _ptr(dXs),
                                          ctypes.c_int(1 if accumulate else 0), _stream(stream)))

    def dr_spmm_plan_destroy(self) -> None:
        if self._p:
            _check(load().dr_spmm_plan_destroy(self._p))
            self._p = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.dr_spmm_plan_destroy()
        except Exception:
            pass


class dr_degree_classes(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("t1", "t2", "k1", "k2", "k3")]


def dr_topk_ranked(X: torch.Tensor, k: int, vals: torch.Tensor, idx: torch.Tensor, stream=None) -> None:
    n, D = X.shape
    _check(load().dr_topk_ranked(_ptr(X), ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int32(k), _ptr(vals), _ptr(idx),
                                 _stream(stream)))


def dr_spmm_fwd_adaptive(A: Csr, xr_vals: torch.Tensor, xr_idx: torch.Tensor, D: int, classes: Sequence[int],
                         H: torch.Tensor, stream=None) -> None:
    """classes = (t1, t2, k1, k2, k3)."""
    a, c = A.c(), dr_degree_classes(*[int(v) for v in classes])
    _check(load().dr_spmm_fwd_adaptive(ctypes.byref(a), _ptr(xr_vals), _ptr(xr_idx), ctypes.c_int32(D), ctypes.byref(c),
                                       _ptr(H), _stream(stream)))


def dr_degree_edge_classes(At: Csr, A_rowptr: torch.Tensor, classes: Sequence[int], edge_class: torch.Tensor,
                           stream=None) -> None:
    a, c = At.c(), dr_degree_classes(*[int(v) for v in classes])
    _check(load().dr_degree_edge_classes(ctypes.byref(a), _ptr(A_rowptr), ctypes.byref(c), _ptr(edge_class), _stream(stream)))


def dr_spmm_bwd_adaptive(At: Csr, edge_class: torch.Tensor, dH: torch.Tensor, xr_idx: torch.Tensor, D: int,
                         classes: Sequence[int], dXr: torch.Tensor, accumulate: bool = False, stream=None) -> None:
    a, c = At.c(), dr_degree_classes(*[int(v) for v in classes])
    _check(load().dr_spmm_bwd_adaptive(ctypes.byref(a), _ptr(edge_class), _ptr(dH), _ptr(xr_idx), ctypes.c_int32(D),
                                       ctypes.byref(c), _ptr(dXr), ctypes.c_int(1 if accumulate else 0), _stream(stream)))


def dr_csr_transpose_workspace_bytes(n_rows: int, n_cols: int, nnz: int) -> int:
    return int(load().dr_csr_transpose_workspace_bytes(ctypes.c_int64(n_rows), ctypes.c_int64(n_cols),
                                                       ctypes.c_int64(nnz)))


def dr_csr_transpose(A: Csr, t_rowptr: torch.Tensor, t_colidx: torch.Tensor, t_vals: Optional[torch.Tensor],
                     workspace: torch.Tensor, stream=None) -> None:
    a = A.c()
    _check(load().dr_csr_transpose(ctypes.byref(a), _ptr(t_rowptr), _ptr(t_colidx), _ptr(t_vals), _ptr(workspace),
                                   ctypes.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream)))


def dr_csr_normalize_workspace_bytes(mode: int, n_rows: int, n_cols: int, nnz: int) -> int:
    return int(load().dr_csr_normalize_workspace_bytes(ctypes.c_int(mode), ctypes.c_int64(n_rows),
                                                       ctypes.c_int64(n_cols), ctypes.c_int64(nnz)))


def dr_csr_normalize(mode: int, n_rows: int, n_cols: int, rowptr: torch.Tensor, colidx: torch.Tensor,
                     vals_out: torch.Tensor, workspace: Optional[torch.Tensor], stream=None) -> None:
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().dr_csr_normalize(ctypes.c_int(mode), ctypes.c_int64(n_rows), ctypes.c_int64(n_cols),
                                   ctypes.c_int64(colidx.shape[0]), _ptr(rowptr), _ptr(colidx), _ptr(vals_out),
                                   _ptr(workspace), ctypes.c_size_t(wsb), _stream(stream)))


def dr_csr_normalize_noalloc(mode: int, n_rows: int, n_cols: int, rowptr: torch.Tensor, colidx: torch.Tensor,
                             vals_out: torch.Tensor, stream=None) -> None:
    _check(load().dr_csr_normalize_noalloc(ctypes.c_int(mode), ctypes.c_int64(n_rows), ctypes.c_int64(n_cols),
                                           ctypes.c_int64(colidx.shape[0]), _ptr(rowptr), _ptr(colidx), _ptr(vals_out),
                                           _stream(stream)))


class HeteroConv:
    """Owner of a ``dr_heteroconv*`` context (heteroconv_create / heteroconv_destroy)."""

    def __init__(self, near: Csr, pins: Csr, pinned: Csr, D: int, k_cell: Optional[int] = None,
                 k_net: Optional[int] = None, per_relation: Optional[Sequence[int]] = None):
        """Either (k_cell, k_net) -> heteroconv_create, or per_relation = (k_near, k_pins, k_pinned) ->
        heteroconv_create_per_relation."""
        self._keep = (near, pins, pinned)
        self.Nc, self.Nn, self.D = near.n_rows, pins.n_rows, D
        self._ctx = ctypes.c_void_p(0)
        a, b, c = near.c(), pins.c(), pinned.c()
        if per_relation is not None:
            if k_cell is not None or k_net is not None:
                raise ValueError("give either (k_cell, k_net) or per_relation")
            kn, kp, kq = (int(v) for v in per_relation)
            _check(load().heteroconv_create_per_relation(
                ctypes.byref(self._ctx), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.c_int32(D),
                ctypes.c_int32(kn), ctypes.c_int32(kp), ctypes.c_int32(kq)))
        else:
            _check(load().heteroconv_create(ctypes.byref(self._ctx), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c),
                                            ctypes.c_int32(D), ctypes.c_int32(k_cell), ctypes.c_int32(k_net)))
        self.k_near, self.k_pins, self.k_self, self.k_pinned = self.heteroconv_get_k()
        self.k_cell, self.k_net = self.k_near, self.k_pinned

    def heteroconv_get_k(self):
        ks = [ctypes.c_int32(0) for _ in range(4)]
        _check(load().heteroconv_get_k(self._ctx, *[ctypes.byref(v) for v in ks]))
        return tuple(int(v.value) for v in ks)

    def heteroconv_profile_k(self, X_cell, X_net, candidates: Sequence[int], warmup: int = 2, reps: int = 5):
        """Returns (ms_fwd[3][n], ms_bwd[3][n], best_k) as nested lists / a tuple (synchronises the device)."""
        n = len(candidates)
        cand = (ctypes.c_int32 * n)(*[int(k) for k in candidates])
        f, b = (ctypes.c_float * (3 * n))(), (ctypes.c_float * (3 * n))()
        best = (ctypes.c_int32 * 3)()
        _check(load().heteroconv_profile_k(self._ctx, _ptr(X_cell), _ptr(X_net), cand, ctypes.c_int32(n),
                                           ctypes.c_int32(warmup), ctypes.c_int32(reps), f, b, best))
        tab = lambda a: [[float(a[r * n + i]) for i in range(n)] for r in range(3)]
        return tab(f), tab(b), tuple(int(v) for v in best)

    def alloc_saved(self, device="cuda") -> Dict[str, torch.Tensor]:
        Nc, Nn, D = self.Nc, self.Nn, self.D
        f32, dev = torch.float32, device
        out = dict(
            vals_cell=torch.empty((Nc, self.k_near), dtype=f32, device=dev),
            idx_cell=torch.empty((Nc, self.k_near), dtype=torch.int16, device=dev),
            vals_net=torch.empty((Nn, self.k_pinned), dtype=f32, device=dev),
            idx_net=torch.empty((Nn, self.k_pinned), dtype=torch.int16, device=dev),
            H_near=torch.empty((Nc, D), dtype=f32, device=dev),
            H_pins=torch.empty((Nn, D), dtype=f32, device=dev),
            H_pinned=torch.empty((Nc, D), dtype=f32, device=dev),
            mask=torch.empty((Nc, D), dtype=torch.uint8, device=dev),
        )
        if self.k_pins != self.k_near:
            out["vals_cell_pins"] = torch.empty((Nc, self.k_pins), dtype=f32, device=dev)
            out["idx_cell_pins"] = torch.empty((Nc, self.k_pins), dtype=torch.int16, device=dev)
        if self.k_self != self.k_pinned:
            out["vals_net_self"] = torch.empty((Nn, self.k_self), dtype=f32, device=dev)
            out["idx_net_self"] = torch.empty((Nn, self.k_self), dtype=torch.int16, device=dev)
        return out

    @staticmethod
    def _saved(saved: Dict[str, torch.Tensor]) -> dr_heteroconv_saved:
        return dr_heteroconv_saved(*[saved[n].data_ptr() if saved.get(n) is not None else 0
                                     for n, _ in dr_heteroconv_saved._fields_])

    @staticmethod
    def _weights(W: Dict[str, torch.Tensor]) -> dr_heteroconv_weights:
        return dr_heteroconv_weights(*[W[n].data_ptr() for n in WEIGHT_NAMES])

    def heteroconv_fwd(self, X_cell, X_net, W, Y_cell, Y_net, saved, stream=None) -> None:
        w, s = self._weights(W), self._saved(saved)
        _check(load().heteroconv_fwd(self._ctx, _ptr(X_cell), _ptr(X_net), ctypes.byref(w), _ptr(Y_cell),
                                     _ptr(Y_net), ctypes.byref(s), _stream(stream)))

    def heteroconv_bwd(self, dY_cell, dY_net, W, saved, dX_cell, dX_net, dW, stream=None) -> None:
        w, s, g = self._weights(W), self._saved(saved), self._weights(dW)
        _check(load().heteroconv_bwd(self._ctx, _ptr(dY_cell), _ptr(dY_net), ctypes.byref(w), ctypes.byref(s),
                                     _ptr(dX_cell), _ptr(dX_net), ctypes.byref(g), _stream(stream)))

    def heteroconv_get_transpose(self, which: int) -> dr_csr:
        out = dr_csr()
        _check(load().heteroconv_get_transpose(self._ctx, ctypes.c_int(which), ctypes.byref(out)))
        return out

    def heteroconv_set_cell_order(self, cell_order: Optional[torch.Tensor], stream=None) -> bool:
        """True when the transposed `near` DR-SpMM of the backward will run on LDS-staged tiles."""
        staged = ctypes.c_int(0)
        _check(load().heteroconv_set_cell_order(self._ctx, _ptr(cell_order), ctypes.byref(staged), _stream(stream)))
        return bool(staged.value)

    def heteroconv_set_overlap(self, mode: int) -> None:
        _check(load().heteroconv_set_overlap(self._ctx, ctypes.c_int(mode)))

    def heteroconv_profile(self, enable: bool) -> None:
        _check(load().heteroconv_profile(self._ctx, ctypes.c_int(1 if enable else 0)))

    def heteroconv_kernel_times(self) -> Dict[str, tuple]:
        """{kernel name: (total ms, launches)} since the previous call (synchronises the device)."""
        lib = load()
        n = int(lib.heteroconv_num_kernels())
        ms = (ctypes.c_double * n)()
        cnt = (ctypes.c_int64 * n)()
        _check(lib.heteroconv_kernel_times(self._ctx, ms, cnt, ctypes.c_int(n)))
        return {lib.heteroconv_kernel_name(i).decode(): (float(ms[i]), int(cnt[i])) for i in range(n)}

    @classmethod
    def borrowed(cls, ctx: int, Nc: int, Nn: int, D: int, keep=None) -> "HeteroConv":
        """A view of a context some other object owns (a pipeline slot): same calls, never destroyed from here."""
        self = cls.__new__(cls)
        self._keep, self._borrowed = keep, True
        self.Nc, self.Nn, self.D = Nc, Nn, D
        self._ctx = ctypes.c_void_p(ctx)
        self.k_near, self.k_pins, self.k_self, self.k_pinned = self.heteroconv_get_k()
        self.k_cell, self.k_net = self.k_near, self.k_pinned
        return self

    def heteroconv_destroy(self) -> None:
        if self._ctx and not getattr(self, "_borrowed", False):
            _check(load().heteroconv_destroy(self._ctx))
        self._ctx = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.heteroconv_destroy()
        except Exception:
            pass


class dr_host_graph(ctypes.Structure):
    _fields_ = [("n_cells", ctypes.c_int64), ("n_nets", ctypes.c_int64), ("nnz_near", ctypes.c_int64),
                ("nnz_pins", ctypes.c_int64), ("near_rowptr", ctypes.c_void_p), ("near_colidx", ctypes.c_void_p),
                ("pins_rowptr", ctypes.c_void_p), ("pins_colidx", ctypes.c_void_p), ("X_cell", ctypes.c_void_p),
                ("X_net", ctypes.c_void_p)]


class Pipeline:
    """Owner of a ``dr_pipeline*`` (dr_pipeline_create / dr_pipeline_destroy).  Host arrays are numpy arrays
    (int32 / float32, C-contiguous); they are kept alive here from submit until acquire."""

    def __init__(self, n_slots: int, n_threads: int, max_cells: int, max_nets: int, max_nnz_near: int,
                 max_nnz_pins: int, D: int, k_cell: int, k_net: int):
        self.D = D
        self._pending = {}
        self._p = ctypes.c_void_p(0)
        _check(load().dr_pipeline_create(ctypes.byref(self._p), ctypes.c_int32(n_slots), ctypes.c_int32(n_threads),
                                         ctypes.c_int64(max_cells), ctypes.c_int64(max_nets),
                                         ctypes.c_int64(max_nnz_near), ctypes.c_int64(max_nnz_pins), ctypes.c_int32(D),
                                         ctypes.c_int32(k_cell), ctypes.c_int32(k_net)))

    def dr_pipeline_submit(self, slot: int, near_rowptr, near_colidx, pins_rowptr, pins_colidx, X_cell=None,
                           X_net=None) -> None:
        import numpy as np
        arrs = [np.ascontiguousarray(a, dtype=np.int32) for a in (near_rowptr, near_colidx, pins_rowptr, pins_colidx)]
        feats = [None if a is None else np.ascontiguousarray(a, dtype=np.float32) for a in (X_cell, X_net)]
        g = dr_host_graph(arrs[0].shape[0] - 1, arrs[2].shape[0] - 1, arrs[1].shape[0], arrs[3].shape[0],
                          *[a.ctypes.data for a in arrs], *[0 if a is None else a.ctypes.data for a in feats])
        _check(load().dr_pipeline_submit(self._p, ctypes.c_int32(slot), ctypes.byref(g)))
        self._pending[slot] = (arrs, feats, g)

    def dr_pipeline_acquire(self, slot: int, stream=None):
        """Returns (HeteroConv view of the slot's context, X_cell device address or None, X_net ... or None)."""
        ctx, xc, xn = ctypes.c_void_p(0), ctypes.c_void_p(0), ctypes.c_void_p(0)
        try:
            _check(load().dr_pipeline_acquire(self._p, ctypes.c_int32(slot), _stream(stream), ctypes.byref(ctx),
                                              ctypes.byref(xc), ctypes.byref(xn)))
        finally:
            arrs, feats, g = self._pending.pop(slot, (None, None, None))
        layer = HeteroConv.borrowed(ctx.value, int(g.n_cells), int(g.n_nets), self.D, keep=self)
        return layer, xc.value, xn.value

    def dr_pipeline_relations(self, slot: int):
        out = (dr_csr * 3)()
        _check(load().dr_pipeline_relations(self._p, ctypes.c_int32(slot), out))
        return [out[i] for i in range(3)]

    def dr_pipeline_release(self, slot: int, stream=None) -> None:
        _check(load().dr_pipeline_release(self._p, ctypes.c_int32(slot), _stream(stream)))

    def dr_pipeline_destroy(self) -> None:
        if self._p:
            _check(load().dr_pipeline_destroy(self._p))
            self._p = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.dr_pipeline_destroy()
        except Exception:
            pass


class dr_hgnn_layer_buffers(ctypes.Structure):
    _fields_ = [("X_cell", ctypes.c_void_p), ("X_net", ctypes.c_void_p), ("Y_cell", ctypes.c_void_p),
                ("Y_net", ctypes.c_void_p), ("saved", dr_heteroconv_saved), ("dY_cell", ctypes.c_void_p),
                ("dY_net", ctypes.c_void_p), ("dX_cell", ctypes.c_void_p), ("dX_net", ctypes.c_void_p),
                ("dW", dr_heteroconv_weights)]


def hgnn_num_params(n_layers: int, D: int) -> int:
    return int(load().hgnn_num_params(ctypes.c_int32(n_layers), ctypes.c_int32(D)))


def _view(ptr: int, shape, dtype) -> torch.Tensor:
    """Copy of a library-owned device buffer as a tensor (device-to-device through the HIP runtime)."""
    t = torch.empty(shape, dtype=dtype, device="cuda")
    if t.numel():
        rc = hip_runtime().hipMemcpy(ctypes.c_void_p(t.data_ptr()), ctypes.c_void_p(ptr),
                                     ctypes.c_size_t(t.numel() * t.element_size()), ctypes.c_int(3))
        if rc != 0:
            raise RuntimeError(f"hipMemcpy failed with {rc}")
    return t


class Hgnn:
    """Owner of a ``dr_hgnn*`` model state (hgnn_create / hgnn_destroy) over a batch of sub-graph contexts."""

    def __init__(self, graphs: Sequence["HeteroConv"], n_layers: int, batched: bool = False):
        """batched=False -> hgnn_create (one stream per sub-graph); True -> hgnn_create_batched (one stacked graph)."""
        self._graphs = list(graphs)
        self.n_layers, self.D, self.batched = n_layers, graphs[0].D, batched
        self._model = ctypes.c_void_p(0)
        arr = (ctypes.c_void_p * len(graphs))(*[g._ctx.value for g in graphs])
        create = load().hgnn_create_batched if batched else load().hgnn_create
        _check(create(ctypes.byref(self._model), ctypes.c_int32(len(graphs)), arr, ctypes.c_int32(n_layers)))

    def hgnn_train_step(self, X_cell, X_net, target, theta, adam_m, adam_v, lr, beta1, beta2, eps, weight_decay, step,
                        grad_out, loss_out, stream=None) -> None:
        n = len(self._graphs)
        tabs = [(ctypes.c_void_p * n)(*[t if isinstance(t, int) else t.data_ptr() for t in lst]) for lst in (X_cell, X_net, target)]
        _check(load().hgnn_train_step(self._model, tabs[0], tabs[1], tabs[2], _ptr(theta), _ptr(adam_m), _ptr(adam_v),
                                      ctypes.c_double(lr), ctypes.c_double(beta1), ctypes.c_double(beta2),
                                      ctypes.c_double(eps), ctypes.c_double(weight_decay), ctypes.c_int32(step),
                                      _ptr(grad_out), _ptr(loss_out), _stream(stream)))

    def hgnn_set_inspection(self, enable: bool) -> None:
        _check(load().hgnn_set_inspection(self._model, ctypes.c_int(1 if enable else 0)))

    def hgnn_get_layer_buffers(self, graph: int, layer: int) -> Dict[str, torch.Tensor]:
        """Copies of the model's buffers for one sub-graph and layer (synchronises)."""
        torch.cuda.synchronize()
        b = dr_hgnn_layer_buffers()
        pred, dpred = ctypes.c_void_p(0), ctypes.c_void_p(0)
        _check(load().hgnn_get_layer_buffers(self._model, ctypes.c_int32(graph), ctypes.c_int32(layer), ctypes.byref(b),
                                             ctypes.byref(pred), ctypes.byref(dpred)))
        g = self._graphs[graph]
        Nc, Nn, D = g.Nc, g.Nn, self.D
        f32 = torch.float32
        out = dict(
            X_cell=_view(b.X_cell, (Nc, D), f32), X_net=_view(b.X_net, (Nn, D), f32),
            Y_cell=_view(b.Y_cell, (Nc, D), f32), Y_net=None if not b.Y_net else _view(b.Y_net, (Nn, D), f32),
            dY_cell=_view(b.dY_cell, (Nc, D), f32), dY_net=_view(b.dY_net, (Nn, D), f32),
            dX_cell=None if not b.dX_cell else _view(b.dX_cell, (Nc, D), f32),
            dX_net=None if not b.dX_net else _view(b.dX_net, (Nn, D), f32),
            pred=_view(pred.value, (Nc,), f32), dpred=_view(dpred.value, (Nc,), f32),
            vals_cell=_view(b.saved.vals_cell, (Nc, g.k_near), f32),
            idx_cell=_view(b.saved.idx_cell, (Nc, g.k_near), torch.int16),
            vals_net=_view(b.saved.vals_net, (Nn, g.k_pinned), f32),
            idx_net=_view(b.saved.idx_net, (Nn, g.k_pinned), torch.int16),
            H_near=_view(b.saved.H_near, (Nc, D), f32),
            H_pins=None if not b.saved.H_pins else _view(b.saved.H_pins, (Nn, D), f32),
            H_pinned=_view(b.saved.H_pinned, (Nc, D), f32), mask=_view(b.saved.mask, (Nc, D), torch.uint8),
        )
        if g.k_pins != g.k_near:
            out["vals_cell_pins"] = _view(b.saved.vals_cell_pins, (Nc, g.k_pins), f32)
            out["idx_cell_pins"] = _view(b.saved.idx_cell_pins, (Nc, g.k_pins), torch.int16)
        if g.k_self != g.k_pinned:
            out["vals_net_self"] = _view(b.saved.vals_net_self, (Nn, g.k_self), f32)
            out["idx_net_self"] = _view(b.saved.idx_net_self, (Nn, g.k_self), torch.int16)
        out["dW"] = {n: _view(getattr(b.dW, n), (D, D), f32) for n in WEIGHT_NAMES}
        return out

    def hgnn_destroy(self) -> None:
        if self._model:
            _check(load().hgnn_destroy(self._model))
            self._model = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.hgnn_destroy()
        except Exception:
            pass
