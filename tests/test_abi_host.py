"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the header
declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2508_16769_amd as P
from paper_2508_16769_amd.binding import dr_csr

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dr_circuitgnn.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(?:int|int64_t|size_t|const char\*)\s+((?:dr_|heteroconv_|hgnn_)\w+)\s*\(", text)
    return sorted(set(names))


def test_header_functions_are_exported_and_bound():
    lib = P.load()
    names = declared_functions()
    assert len(names) >= 19
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"
    assert sorted(P.EXPORTS) == names
    assert P.dr_abi_version() == 2


def _null_csr(n_rows=4, n_cols=4, nnz=0, rowptr=8, colidx=8, vals=8):
    return dr_csr(n_rows, n_cols, nnz, rowptr, colidx, vals)


def test_topk_argument_errors():
    lib = P.load()
    one = ctypes.c_void_p(16)
    assert lib.dr_topk(one, ctypes.c_int64(4), 8, 9, one, one, None) == P.DR_ERR_INVALID_ARG
    assert "exceeds D" in P.dr_last_error()
    assert lib.dr_topk(one, ctypes.c_int64(4), 8, 0, one, one, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_topk(one, ctypes.c_int64(4), 0, 1, one, one, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_topk(one, ctypes.c_int64(-1), 8, 2, one, one, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_topk(None, ctypes.c_int64(4), 8, 2, one, one, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_topk(one, ctypes.c_int64(4), 2048, 2, one, one, None) == P.DR_ERR_UNSUPPORTED
    assert lib.dr_topk(ctypes.c_void_p(18), ctypes.c_int64(4), 8, 2, one, one, None) == P.DR_ERR_INVALID_ARG
    assert "misaligned" in P.dr_last_error()
    # n == 0 is a no-op that never touches the GPU
    assert lib.dr_topk(None, ctypes.c_int64(0), 8, 2, None, None, None) == P.DR_OK


def test_spmm_argument_errors():
    lib = P.load()
    one = ctypes.c_void_p(16)
    A = _null_csr(nnz=3)
    assert lib.dr_spmm_fwd(None, one, one, 8, 2, one, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_spmm_fwd(ctypes.byref(A), one, one, 8, 9, one, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_spmm_fwd(ctypes.byref(A), one, one, 8, 2, None, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_spmm_fwd(ctypes.byref(A), None, one, 8, 2, one, None) == P.DR_ERR_INVALID_ARG
    B = _null_csr(nnz=3, vals=0)
    assert lib.dr_spmm_fwd(ctypes.byref(B), one, one, 8, 2, one, None) == P.DR_ERR_INVALID_ARG
    assert "null vals" in P.dr_last_error()
    C = _null_csr(nnz=2 ** 31)
    assert lib.dr_spmm_fwd(ctypes.byref(C), one, one, 8, 2, one, None) == P.DR_ERR_INVALID_ARG
    assert "nnz" in P.dr_last_error()
    Z = _null_csr(n_rows=0)
    assert lib.dr_spmm_fwd(ctypes.byref(Z), None, None, 8, 2, None, None) == P.DR_OK
    assert lib.dr_spmm_bwd(ctypes.byref(A), one, one, 8, 9, one, 0, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_spmm_bwd(ctypes.byref(A), None, one, 8, 2, one, 0, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_spmm_bwd(ctypes.byref(A), one, None, 8, 2, one, 0, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_spmm_bwd(ctypes.byref(Z), None, None, 8, 2, None, 0, None) == P.DR_OK


def test_setup_argument_errors_and_workspace_sizes():
    lib = P.load()
    one = ctypes.c_void_p(256)
    A = _null_csr(nnz=5, rowptr=256, colidx=256, vals=256)
    need = P.dr_csr_transpose_workspace_bytes(4, 4, 5)
    assert need >= 4 * (4 + 5 + 5) and need % 256 == 0
    assert lib.dr_csr_transpose(ctypes.byref(A), one, one, one, one, ctypes.c_size_t(need - 1), None) \
        == P.DR_ERR_WORKSPACE
    assert lib.dr_csr_transpose(ctypes.byref(A), one, one, one, None, ctypes.c_size_t(need), None) \
        == P.DR_ERR_INVALID_ARG
    assert lib.dr_csr_transpose(ctypes.byref(A), one, one, None, one, ctypes.c_size_t(need), None) \
        == P.DR_ERR_INVALID_ARG
    assert lib.dr_csr_transpose(ctypes.byref(A), one, one, one, ctypes.c_void_p(260), ctypes.c_size_t(need), None) \
        == P.DR_ERR_INVALID_ARG
    assert P.dr_csr_normalize_workspace_bytes(P.DR_NORM_MEAN, 4, 4, 5) == 0
    assert P.dr_csr_normalize_workspace_bytes(P.DR_NORM_SYM, 4, 1000, 5) >= 4000
    i64 = ctypes.c_int64
    assert lib.dr_csr_normalize(7, i64(4), i64(4), i64(5), one, one, one, None, ctypes.c_size_t(0), None) \
        == P.DR_ERR_INVALID_ARG
    assert lib.dr_csr_normalize(P.DR_NORM_SYM, i64(4), i64(4), i64(5), one, one, one, one, ctypes.c_size_t(4), None) \
        == P.DR_ERR_WORKSPACE
    assert lib.dr_csr_normalize(P.DR_NORM_MEAN, i64(4), i64(4), i64(5), one, one, None, None, ctypes.c_size_t(0),
                                None) == P.DR_ERR_INVALID_ARG


def test_heteroconv_create_argument_errors():
    lib = P.load()
    ctx = ctypes.c_void_p(0)
    near = _null_csr(8, 8, 3)
    pins = _null_csr(5, 8, 3)
    pinned = _null_csr(8, 5, 3)
    bad = _null_csr(8, 6, 3)
    r = lib.heteroconv_create(ctypes.byref(ctx), ctypes.byref(near), ctypes.byref(pins), ctypes.byref(bad), 64, 16, 16)
    assert r == P.DR_ERR_INVALID_ARG and "pinned must be" in P.dr_last_error()
    r = lib.heteroconv_create(ctypes.byref(ctx), ctypes.byref(near), ctypes.byref(pins), ctypes.byref(pinned), 64, 65, 16)
    assert r == P.DR_ERR_INVALID_ARG
    r = lib.heteroconv_create(ctypes.byref(ctx), ctypes.byref(near), ctypes.byref(pins), ctypes.byref(pinned), 80, 16, 16)
    assert r == P.DR_ERR_UNSUPPORTED
    r = lib.heteroconv_create(None, ctypes.byref(near), ctypes.byref(pins), ctypes.byref(pinned), 64, 16, 16)
    assert r == P.DR_ERR_INVALID_ARG
    assert lib.heteroconv_destroy(None) == P.DR_OK


def test_newer_entry_points_validate_on_the_host():
    """Per-relation K, K profiling, adaptive K, the batched model and the pipeline: argument errors come back before any
    HIP call (this test runs without a GPU)."""
    from paper_2508_16769_amd.binding import dr_degree_classes, dr_host_graph
    lib = P.load()
    one = ctypes.c_void_p(16)
    i64 = ctypes.c_int64
    ctx = ctypes.c_void_p(0)
    near, pins, pinned = _null_csr(8, 8, 3), _null_csr(5, 8, 3), _null_csr(8, 5, 3)
    args = (ctypes.byref(ctx), ctypes.byref(near), ctypes.byref(pins), ctypes.byref(pinned))
    assert lib.heteroconv_create_per_relation(*args, 64, 16, 0, 16) == P.DR_ERR_INVALID_ARG
    assert lib.heteroconv_create_per_relation(*args, 64, 16, 16, 65) == P.DR_ERR_INVALID_ARG
    assert lib.heteroconv_create_per_relation(*args, 48, 16, 16, 16) == P.DR_ERR_UNSUPPORTED
    assert lib.heteroconv_profile_k(None, one, one, one, 1, 0, 1, one, one, one) == P.DR_ERR_INVALID_ARG
    assert lib.heteroconv_get_k(None, one, one, one, one) == P.DR_ERR_INVALID_ARG
    # adaptive K
    A = _null_csr(nnz=3)
    for bad in ((3, 2, 8, 4, 2), (-1, 2, 8, 4, 2), (1, 2, 4, 8, 2), (1, 2, 8, 4, 0), (1, 2, 9, 4, 2)):
        c = dr_degree_classes(*bad)
        assert lib.dr_spmm_fwd_adaptive(ctypes.byref(A), one, one, 8, ctypes.byref(c), one, None) == P.DR_ERR_INVALID_ARG, bad
        assert lib.dr_spmm_bwd_adaptive(ctypes.byref(A), one, one, one, 8, ctypes.byref(c), one, 0, None) == P.DR_ERR_INVALID_ARG, bad
    wide = dr_degree_classes(1, 2, 96, 4, 2)
    assert lib.dr_spmm_fwd_adaptive(ctypes.byref(A), one, one, 128, ctypes.byref(wide), one, None) == P.DR_ERR_UNSUPPORTED
    ok = dr_degree_classes(1, 2, 8, 4, 2)
    assert lib.dr_spmm_fwd_adaptive(ctypes.byref(A), one, one, 8, None, one, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_spmm_fwd_adaptive(ctypes.byref(A), None, one, 8, ctypes.byref(ok), one, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_spmm_bwd_adaptive(ctypes.byref(A), None, one, one, 8, ctypes.byref(ok), one, 0, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_degree_edge_classes(ctypes.byref(A), None, ctypes.byref(ok), one, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_topk_ranked(one, i64(4), 8, 9, one, one, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_topk_ranked(None, i64(0), 8, 2, None, None, None) == P.DR_OK
    # batched model and pipeline
    mdl = ctypes.c_void_p(0)
    assert lib.hgnn_create_batched(ctypes.byref(mdl), 0, None, 2) == P.DR_ERR_INVALID_ARG
    assert lib.hgnn_create_batched(ctypes.byref(mdl), 1, None, 2) == P.DR_ERR_INVALID_ARG
    pl = ctypes.c_void_p(0)
    assert lib.dr_pipeline_create(ctypes.byref(pl), 0, 1, i64(10), i64(10), i64(10), i64(10), 64, 16, 16) == P.DR_ERR_INVALID_ARG
    assert lib.dr_pipeline_create(ctypes.byref(pl), 1, 99, i64(10), i64(10), i64(10), i64(10), 64, 16, 16) == P.DR_ERR_INVALID_ARG
    assert lib.dr_pipeline_create(ctypes.byref(pl), 1, 1, i64(0), i64(10), i64(10), i64(10), 64, 16, 16) == P.DR_ERR_INVALID_ARG
    assert lib.dr_pipeline_create(None, 1, 1, i64(10), i64(10), i64(10), i64(10), 64, 16, 16) == P.DR_ERR_INVALID_ARG
    g = dr_host_graph()
    assert lib.dr_pipeline_submit(None, 0, ctypes.byref(g)) == P.DR_ERR_INVALID_ARG
    assert lib.dr_pipeline_acquire(None, 0, None, ctypes.byref(ctx), None, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_pipeline_release(None, 0, None) == P.DR_ERR_INVALID_ARG
    assert lib.dr_pipeline_destroy(None) == P.DR_OK


def test_binding_refuses_missing_library(monkeypatch, tmp_path):
    """No CPU fallback: if the shared library cannot be loaded the binding raises."""
    from paper_2508_16769_amd import binding, build
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(build, "LIB", str(tmp_path / "missing" / "libdrcgnn.so"))
    monkeypatch.setattr(build, "build", lambda verbose=False: (_ for _ in ()).throw(RuntimeError("no hipcc")))
    with pytest.raises(RuntimeError):
        binding.load()
