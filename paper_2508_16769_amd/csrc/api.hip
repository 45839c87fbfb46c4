// C ABI entry points: host-side argument validation, then the kernel launchers.
#include "dr_internal.h"

#include <cstring>

namespace drc {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char* what) {
    snprintf(g_err, sizeof(g_err), "HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
    return DR_ERR_HIP;
}

int check_csr(const dr_csr* A, const char* name, bool need_vals) {
    DRC_REQUIRE(A != nullptr, "%s: null dr_csr", name);
    DRC_REQUIRE(A->n_rows >= 0 && A->n_cols >= 0 && A->nnz >= 0, "%s: negative dimension", name);
    DRC_REQUIRE(A->n_rows < (int64_t(1) << 31) - 1 && A->n_cols < (int64_t(1) << 31) - 1,
                "%s: more than 2^31-2 rows or columns", name);
    DRC_REQUIRE(A->nnz < (int64_t(1) << 31), "%s: nnz >= 2^31", name);
    DRC_REQUIRE(A->rowptr != nullptr, "%s: null rowptr", name);
    DRC_REQUIRE(A->nnz == 0 || A->colidx != nullptr, "%s: null colidx", name);
    DRC_REQUIRE(!need_vals || A->nnz == 0 || A->vals != nullptr, "%s: null vals", name);
    DRC_REQUIRE(A->nnz == 0 || A->n_cols > 0, "%s: edges but no columns", name);
    return DR_OK;
}

static int check_dk(int32_t D, int32_t k, const char* fn) {
    DRC_REQUIRE(D >= 1, "%s: D must be >= 1 (got %d)", fn, D);
    DRC_REQUIRE(k >= 1, "%s: k must be >= 1 (got %d)", fn, k);
    DRC_REQUIRE(k <= D, "%s: k (%d) exceeds D (%d)", fn, k, D);
    if (D > DR_MAX_D) return fail(DR_ERR_UNSUPPORTED, "%s: D = %d exceeds DR_MAX_D = %d", fn, D, DR_MAX_D);
    return DR_OK;
}

}  // namespace drc

using namespace drc;

extern "C" {

const char* dr_last_error(void) { return g_err; }

int dr_abi_version(void) { return 2; }

int dr_topk(const float* X, int64_t n, int32_t D, int32_t k, float* vals, uint16_t* idx, void* stream) {
    if (int rc = check_dk(D, k, "dr_topk")) return rc;
    DRC_REQUIRE(n >= 0, "dr_topk: negative row count");
    DRC_REQUIRE(n < (int64_t(1) << 31), "dr_topk: more than 2^31-1 rows");
    if (n == 0) return DR_OK;
    DRC_REQUIRE(X && vals && idx, "dr_topk: null pointer");
    DRC_REQUIRE(aligned(X, 4) && aligned(vals, 4) && aligned(idx, 2), "dr_topk: misaligned pointer");
    return launch_topk(X, n, D, k, vals, idx, as_stream(stream));
}

int dr_spmm_fwd(const dr_csr* A, const float* xs_vals, const uint16_t* xs_idx, int32_t D, int32_t k, float* H,
                void* stream) {
    if (int rc = check_csr(A, "dr_spmm_fwd: A", true)) return rc;
    if (int rc = check_dk(D, k, "dr_spmm_fwd")) return rc;
    if (A->n_rows == 0) return DR_OK;
    DRC_REQUIRE(H != nullptr, "dr_spmm_fwd: null H");
    DRC_REQUIRE(A->nnz == 0 || (xs_vals && xs_idx), "dr_spmm_fwd: null CBSR operand");
    DRC_REQUIRE(aligned(H, 4) && aligned(xs_vals, 4) && aligned(xs_idx, 2), "dr_spmm_fwd: misaligned pointer");
    DRC_REQUIRE(A->n_cols * (int64_t)k < (int64_t(1) << 31), "dr_spmm_fwd: N*k >= 2^31");
    return launch_spmm_fwd(A, xs_vals, xs_idx, D, k, H, as_stream(stream));
}

int dr_spmm_bwd(const dr_csr* At, const float* dH, const uint16_t* xs_idx, int32_t D, int32_t k, float* dXs,
                int accumulate, void* stream) {
    if (int rc = check_csr(At, "dr_spmm_bwd: At", true)) return rc;
    if (int rc = check_dk(D, k, "dr_spmm_bwd")) return rc;
    if (At->n_rows == 0) return DR_OK;
    DRC_REQUIRE(dXs != nullptr && xs_idx != nullptr, "dr_spmm_bwd: null dXs or xs_idx");
    DRC_REQUIRE(At->nnz == 0 || dH != nullptr, "dr_spmm_bwd: null dH");
    DRC_REQUIRE(aligned(dH, 4) && aligned(dXs, 4) && aligned(xs_idx, 2), "dr_spmm_bwd: misaligned pointer");
    DRC_REQUIRE(At->n_cols * (int64_t)D < (int64_t(1) << 32), "dr_spmm_bwd: M*D >= 2^32");
    return launch_spmm_bwd(At, dH, xs_idx, D, k, dXs, accumulate, as_stream(stream));
}

static int check_classes(const dr_degree_classes* c, int32_t D, const char* fn) {
    DRC_REQUIRE(c != nullptr, "%s: null degree classes", fn);
    DRC_REQUIRE(c->t1 >= 0 && c->t1 <= c->t2, "%s: class boundaries must satisfy 0 <= t1 <= t2 (got %d, %d)", fn, c->t1, c->t2);
    DRC_REQUIRE(c->k3 >= 1 && c->k2 >= c->k3 && c->k1 >= c->k2, "%s: widths must satisfy k1 >= k2 >= k3 >= 1 (got %d, %d, %d)", fn,
                c->k1, c->k2, c->k3);
    if (int rc = check_dk(D, c->k1, fn)) return rc;
    if (c->k1 > 64) return fail(DR_ERR_UNSUPPORTED, "%s: k1 = %d exceeds 64", fn, c->k1);
    return DR_OK;
}

int dr_topk_ranked(const float* X, int64_t n, int32_t D, int32_t k, float* vals, uint16_t* idx, void* stream) {
    if (int rc = check_dk(D, k, "dr_topk_ranked")) return rc;
    DRC_REQUIRE(n >= 0 && n < (int64_t(1) << 31), "dr_topk_ranked: n out of range");
    if (n == 0) return DR_OK;
    DRC_REQUIRE(X && vals && idx, "dr_topk_ranked: null pointer");
    DRC_REQUIRE(aligned(X, 4) && aligned(vals, 4) && aligned(idx, 2), "dr_topk_ranked: misaligned pointer");
    DRC_REQUIRE(n * (int64_t)D < (int64_t(1) << 33) && n * (int64_t)k < (int64_t(1) << 31), "dr_topk_ranked: n*D or n*k too large");
    return launch_topk_ranked(X, n, D, k, vals, idx, as_stream(stream));
}

int dr_spmm_fwd_adaptive(const dr_csr* A, const float* xr_vals, const uint16_t* xr_idx, int32_t D,
                         const dr_degree_classes* cls, float* H, void* stream) {
    if (int rc = check_csr(A, "dr_spmm_fwd_adaptive: A", true)) return rc;
    if (int rc = check_classes(cls, D, "dr_spmm_fwd_adaptive")) return rc;
    if (A->n_rows == 0) return DR_OK;
    DRC_REQUIRE(H != nullptr, "dr_spmm_fwd_adaptive: null H");
    DRC_REQUIRE(A->nnz == 0 || (xr_vals && xr_idx), "dr_spmm_fwd_adaptive: null CBSR operand");
    DRC_REQUIRE(aligned(H, 4) && aligned(xr_vals, 4) && aligned(xr_idx, 2), "dr_spmm_fwd_adaptive: misaligned pointer");
    DRC_REQUIRE(A->n_cols * (int64_t)cls->k1 < (int64_t(1) << 31), "dr_spmm_fwd_adaptive: N*k1 >= 2^31");
    return launch_spmm_fwd_adaptive(A, xr_vals, xr_idx, D, cls, H, as_stream(stream));
}

int dr_degree_edge_classes(const dr_csr* At, const int32_t* A_rowptr, const dr_degree_classes* cls, uint8_t* edge_class,
                           void* stream) {
    if (int rc = check_csr(At, "dr_degree_edge_classes: At", false)) return rc;
    DRC_REQUIRE(cls != nullptr && cls->t1 >= 0 && cls->t1 <= cls->t2, "dr_degree_edge_classes: class boundaries must satisfy 0 <= t1 <= t2");
    if (At->nnz == 0) return DR_OK;
    DRC_REQUIRE(A_rowptr != nullptr && edge_class != nullptr, "dr_degree_edge_classes: null pointer");
    return launch_edge_classes(At, A_rowptr, cls, edge_class, as_stream(stream));
}

int dr_spmm_bwd_adaptive(const dr_csr* At, const uint8_t* edge_class, const float* dH, const uint16_t* xr_idx, int32_t D,
                         const dr_degree_classes* cls, float* dXr, int accumulate, void* stream) {
    if (int rc = check_csr(At, "dr_spmm_bwd_adaptive: At", true)) return rc;
    if (int rc = check_classes(cls, D, "dr_spmm_bwd_adaptive")) return rc;
    if (At->n_rows == 0) return DR_OK;
    DRC_REQUIRE(dXr != nullptr && xr_idx != nullptr, "dr_spmm_bwd_adaptive: null dXr or xr_idx");
    DRC_REQUIRE(At->nnz == 0 || (dH != nullptr && edge_class != nullptr), "dr_spmm_bwd_adaptive: null dH or edge_class");
    DRC_REQUIRE(aligned(dH, 4) && aligned(dXr, 4) && aligned(xr_idx, 2), "dr_spmm_bwd_adaptive: misaligned pointer");
    DRC_REQUIRE(At->n_cols < (int64_t(1) << 30), "dr_spmm_bwd_adaptive: 2^30 or more destinations");
    DRC_REQUIRE(At->n_cols * (int64_t)D < (int64_t(1) << 32), "dr_spmm_bwd_adaptive: M*D >= 2^32");
    return launch_spmm_bwd_adaptive(At, edge_class, dH, xr_idx, D, cls, dXr, accumulate, as_stream(stream));
}

static size_t align256(size_t b) { return (b + 255) & ~size_t(255); }

size_t dr_csr_transpose_workspace_bytes(int64_t n_rows, int64_t n_cols, int64_t nnz) {
    (void)n_rows;
    if (n_cols < 0 || nnz < 0) return 0;
    // cursor[n_cols] | edge key[nnz] | edge row[nnz] | block sums | counter and list of the rows of more than 64 entries
    return align256(4 * (size_t)(n_cols + 1)) + 2 * align256(4 * (size_t)(nnz + 1)) +
           align256(4 * ((size_t)(n_cols + 1) / 1024 + 2)) + align256(4 * ((size_t)n_cols + 64));
}

int dr_csr_transpose(const dr_csr* A, int32_t* t_rowptr, int32_t* t_colidx, float* t_vals, void* workspace,
                     size_t workspace_bytes, void* stream) {
    if (int rc = check_csr(A, "dr_csr_transpose: A", false)) return rc;
    DRC_REQUIRE(t_rowptr != nullptr, "dr_csr_transpose: null t_rowptr");
    DRC_REQUIRE(A->nnz == 0 || t_colidx != nullptr, "dr_csr_transpose: null t_colidx");
    DRC_REQUIRE((A->vals == nullptr) == (t_vals == nullptr) || A->nnz == 0,
                "dr_csr_transpose: vals and t_vals must both be given or both be NULL");
    size_t need = dr_csr_transpose_workspace_bytes(A->n_rows, A->n_cols, A->nnz);
    DRC_REQUIRE(workspace != nullptr, "dr_csr_transpose: null workspace");
    DRC_REQUIRE(aligned(workspace, 256), "dr_csr_transpose: workspace must be 256-byte aligned");
    if (workspace_bytes < need)
        return fail(DR_ERR_WORKSPACE, "dr_csr_transpose: workspace has %zu bytes, needs %zu", workspace_bytes, need);
    return launch_csr_transpose(A, t_rowptr, t_colidx, t_vals, workspace, as_stream(stream));
}

size_t dr_csr_normalize_workspace_bytes(int mode, int64_t n_rows, int64_t n_cols, int64_t nnz) {
    (void)n_rows;
    (void)nnz;
    if (mode != DR_NORM_SYM || n_cols < 0) return 0;
    return align256(4 * (size_t)(n_cols + 1));
}

int dr_csr_normalize(int mode, int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t* rowptr,
                     const int32_t* colidx, float* vals_out, void* workspace, size_t workspace_bytes,
                     void* stream) {
    DRC_REQUIRE(mode == DR_NORM_MEAN || mode == DR_NORM_SYM, "dr_csr_normalize: unknown mode %d", mode);
    dr_csr A{n_rows, n_cols, nnz, rowptr, colidx, nullptr};
    if (int rc = check_csr(&A, "dr_csr_normalize", false)) return rc;
    if (nnz == 0) return DR_OK;
    DRC_REQUIRE(vals_out != nullptr, "dr_csr_normalize: null vals_out");
    size_t need = dr_csr_normalize_workspace_bytes(mode, n_rows, n_cols, nnz);
    if (need > 0) {
        DRC_REQUIRE(workspace != nullptr, "dr_csr_normalize: null workspace");
        DRC_REQUIRE(aligned(workspace, 256), "dr_csr_normalize: workspace must be 256-byte aligned");
        if (workspace_bytes < need)
            return fail(DR_ERR_WORKSPACE, "dr_csr_normalize: workspace has %zu bytes, needs %zu", workspace_bytes,
                        need);
    }
    return launch_csr_normalize(mode, n_rows, n_cols, nnz, rowptr, colidx, vals_out, workspace, as_stream(stream));
}

int dr_csr_normalize_noalloc(int mode, int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t* rowptr,
                             const int32_t* colidx, float* vals_out, void* stream) {
    DRC_REQUIRE(mode == DR_NORM_MEAN || mode == DR_NORM_SYM, "dr_csr_normalize_noalloc: unknown mode %d", mode);
    dr_csr A{n_rows, n_cols, nnz, rowptr, colidx, nullptr};
    if (int rc = check_csr(&A, "dr_csr_normalize_noalloc", false)) return rc;
    if (nnz == 0) return DR_OK;
    DRC_REQUIRE(vals_out != nullptr, "dr_csr_normalize_noalloc: null vals_out");
    if (mode == DR_NORM_SYM && n_cols > DR_NOALLOC_MAX_COLS)
        return fail(DR_ERR_UNSUPPORTED, "dr_csr_normalize_noalloc: n_cols = %lld exceeds DR_NOALLOC_MAX_COLS = %d",
                    (long long)n_cols, DR_NOALLOC_MAX_COLS);
    return launch_csr_normalize_noalloc(mode, n_rows, n_cols, nnz, rowptr, colidx, vals_out, as_stream(stream));
}

}  // extern "C"
