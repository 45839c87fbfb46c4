"""Device-memory plumbing around the binding: upload a host CSR pattern, attach the module's edge values
(dr_csr_normalize) and transpose on the device (dr_csr_transpose).  PyTorch is used only to own HBM."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _ws(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def upload_pattern(pattern, device="cuda") -> B.Csr:
    """``pattern`` needs n_rows, n_cols, rowptr, colidx (host int32 arrays)."""
    rowptr = torch.from_numpy(np.ascontiguousarray(pattern.rowptr, dtype=np.int32)).to(device)
    colidx = torch.from_numpy(np.ascontiguousarray(pattern.colidx, dtype=np.int32)).to(device)
    return B.Csr(int(pattern.n_rows), int(pattern.n_cols), rowptr, colidx, None)


def device_relation(pattern, mode: int, device="cuda") -> B.Csr:
    """Upload a pattern and fill its edge values on the device (DR_NORM_MEAN or DR_NORM_SYM)."""
    A = upload_pattern(pattern, device)
    A.vals = torch.empty(A.nnz, dtype=torch.float32, device=device)
    ws = _ws(B.dr_csr_normalize_workspace_bytes(mode, A.n_rows, A.n_cols, A.nnz), device)
    B.dr_csr_normalize(mode, A.n_rows, A.n_cols, A.rowptr, A.colidx, A.vals, ws)
    return A


def device_transpose(A: B.Csr) -> B.Csr:
    """Stable transpose on the device; returns a new Csr that owns its arrays."""
    dev = A.rowptr.device
    t_rowptr = torch.empty(A.n_cols + 1, dtype=torch.int32, device=dev)
    t_colidx = torch.empty(A.nnz, dtype=torch.int32, device=dev)
    t_vals = None if A.vals is None else torch.empty(A.nnz, dtype=torch.float32, device=dev)
    ws = _ws(B.dr_csr_transpose_workspace_bytes(A.n_rows, A.n_cols, A.nnz), dev)
    B.dr_csr_transpose(A, t_rowptr, t_colidx, t_vals, ws)
    torch.cuda.current_stream().synchronize()   # workspace is released on return
    return B.Csr(A.n_cols, A.n_rows, t_rowptr, t_colidx, t_vals)
