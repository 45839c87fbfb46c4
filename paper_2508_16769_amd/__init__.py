"""MI355X-native HeteroConv DR-SpMM hot path of DR-CircuitGNN: hand-written HIP kernels behind a C ABI
(``include/dr_circuitgnn.h``, built in-tree as ``libdrcgnn.so``) and a thin ctypes binding of the same names."""
from .binding import (  # noqa: F401
    DR_ERR_HIP, DR_ERR_INVALID_ARG, DR_ERR_UNSUPPORTED, DR_ERR_WORKSPACE, DR_NORM_MEAN, DR_NORM_SYM, DR_OK,
    DR_OVERLAP_AUTO, DR_OVERLAP_OFF, DR_OVERLAP_ON,
    EXPORTS, WEIGHT_NAMES, Csr, DrError, HeteroConv, Hgnn, Pipeline, SpmmPlan, hgnn_num_params,
    dr_abi_version, dr_csr_normalize, dr_csr_normalize_noalloc, dr_csr_normalize_workspace_bytes, dr_csr_transpose,
    dr_csr_transpose_workspace_bytes, dr_degree_edge_classes, dr_last_error, dr_spmm_bwd, dr_spmm_bwd_adaptive, dr_spmm_fwd, dr_spmm_fwd_adaptive, dr_topk, dr_topk_ranked, library_path, load,
)
from .device import device_relation, device_transpose, upload_pattern  # noqa: F401
