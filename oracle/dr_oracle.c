/*
 * CPU oracle for the DR-CircuitGNN HeteroConv hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
 * definition of what the GPU library must compute.  It shares no code with the
 * HIP path and must never be called from it; only the test-suite, the smoke
 * check and the benchmark's cpu_baseline leg load it.
 *
 * Everything floating-point is evaluated in fp64.  Feature / gradient / weight
 * inputs are fp64 arrays (the callers widen their fp32 data exactly); adjacency
 * values are the fp32 numbers the GPU consumes, widened on use.
 *
 * Notation follows the paper: relation psi has adjacency A (M destination rows,
 * N source columns); X is a source embedding [N, D]; f(X) is the row-wise
 * Dynamic-ReLU of X with k survivors per row, stored as CBSR = (vals[N,k],
 * idx[N,k]).
 *
 * Parity pins (see tests, marker "not gpu"): brute-force sort, dense matmul,
 * scipy CSR product, adjoint identity, finite differences, constructed ties.
 * The module formulas of orc_heteroconv_* (SageConv = self + mean-neighbour with
 * two weights, GraphConv = symmetric normalisation with one weight, no bias) are
 * the textbook definitions; the paper does not print them: parity unpinned by the
 * paper for that choice, pinned only to the finite-difference and dense checks.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* D-ReLU: Section 3.1, threshold equation th_i = min(topk(X_i, k)) and the   */
/* piecewise definition of f(X).  Exactly k survivors per row: the k largest  */
/* signed values; among equal values the lower column wins.  Survivors are    */
/* emitted in ascending column order.                                         */
/* ------------------------------------------------------------------------ */

typedef struct { double v; int32_t c; } orc_entry;

static int orc_cmp_value_desc_col_asc(const void* pa, const void* pb) {
    const orc_entry* a = (const orc_entry*)pa;
    const orc_entry* b = (const orc_entry*)pb;
    if (a->v > b->v) return -1;   /* -0.0 and +0.0 compare equal here */
    if (a->v < b->v) return 1;
    return (a->c > b->c) - (a->c < b->c);
}

static int orc_cmp_col_asc(const void* pa, const void* pb) {
    const orc_entry* a = (const orc_entry*)pa;
    const orc_entry* b = (const orc_entry*)pb;
    return (a->c > b->c) - (a->c < b->c);
}

/* returns 0, or -1 on bad arguments / non-finite input */
int orc_topk(const double* X, int64_t n, int32_t D, int32_t k, double* vals, int32_t* idx) {
    if (D < 1 || k < 1 || k > D) return -1;
    orc_entry* row = (orc_entry*)malloc(sizeof(orc_entry) * (size_t)D);
    if (!row) return -1;
    for (int64_t i = 0; i < n; ++i) {
        for (int32_t d = 0; d < D; ++d) {
            double v = X[i * D + d];
            if (!isfinite(v)) { free(row); return -1; }
            row[d].v = v;
            row[d].c = d;
        }
        qsort(row, (size_t)D, sizeof(orc_entry), orc_cmp_value_desc_col_asc);
        qsort(row, (size_t)k, sizeof(orc_entry), orc_cmp_col_asc);
        for (int32_t t = 0; t < k; ++t) {
            vals[i * k + t] = row[t].v;
            idx[i * k + t] = row[t].c;
        }
    }
    free(row);
    return 0;
}

/* f(X) as a dense [n, D] array: the k survivors in place, zeros elsewhere. */
void orc_densify(const double* vals, const int32_t* idx, int64_t n, int32_t D, int32_t k, double* Xd) {
    memset(Xd, 0, sizeof(double) * (size_t)n * (size_t)D);
    for (int64_t i = 0; i < n; ++i)
        for (int32_t t = 0; t < k; ++t)
            Xd[i * D + idx[i * k + t]] = vals[i * k + t];
}

/* ------------------------------------------------------------------------ */
/* Edge values of the three modules (GraphSAGE 'mean' mode, Section 4.1; GCN  */
/* symmetric normalisation).  deg_in(i) = stored entries of row i; deg_out(j) */
/* = stored entries with column j; duplicates count separately.               */
/*   mode 0 (mean): a_ij = 1 / deg_in(i)                                      */
/*   mode 1 (sym) : a_ij = 1 / sqrt(max(deg_in(i),1) * max(deg_out(j),1))     */
/* Evaluated in fp64 and rounded once to fp32 (the SpMM input type).          */
/* ------------------------------------------------------------------------ */
int orc_csr_normalize(int mode, int64_t n_rows, int64_t n_cols, const int32_t* rowptr,
                      const int32_t* colidx, float* vals_out) {
    if (mode == 0) {
        for (int64_t i = 0; i < n_rows; ++i) {
            int32_t b = rowptr[i], e = rowptr[i + 1];
            for (int32_t p = b; p < e; ++p) vals_out[p] = (float)(1.0 / (double)(e - b));
        }
        return 0;
    }
    if (mode == 1) {
        int64_t* deg_out = (int64_t*)calloc((size_t)(n_cols > 0 ? n_cols : 1), sizeof(int64_t));
        if (!deg_out) return -1;
        for (int64_t p = 0; p < rowptr[n_rows]; ++p) deg_out[colidx[p]] += 1;
        for (int64_t i = 0; i < n_rows; ++i) {
            int32_t b = rowptr[i], e = rowptr[i + 1];
            double di = (double)((e - b) > 1 ? (e - b) : 1);
            for (int32_t p = b; p < e; ++p) {
                int64_t o = deg_out[colidx[p]];
                double dj = (double)(o > 1 ? o : 1);
                vals_out[p] = (float)(1.0 / sqrt(di * dj));
            }
        }
        free(deg_out);
        return 0;
    }
    return -1;
}

/* ------------------------------------------------------------------------ */
/* DR-SpMM forward, per-row neighbour aggregation (Section 3.2, Eq. for       */
/* Y_i = sum_j A_ij X_j, with X replaced by f(X) held as CBSR):               */
/*   H[i, c] = sum_{e in row i} a_e * f(X)[col_e, c]                          */
/* l1elem (optional, may be NULL) receives sum |a_e * v| per output element,  */
/* l1row (optional) the same summed over the row.                             */
/* ------------------------------------------------------------------------ */
void orc_spmm_fwd(int64_t M, const int32_t* rowptr, const int32_t* colidx, const float* avals,
                  const double* xs_vals, const int32_t* xs_idx, int32_t D, int32_t k,
                  double* H, double* l1elem, double* l1row) {
    for (int64_t i = 0; i < M; ++i) {
        double* h = H + i * D;
        for (int32_t c = 0; c < D; ++c) h[c] = 0.0;
        if (l1elem) for (int32_t c = 0; c < D; ++c) l1elem[i * D + c] = 0.0;
        double row_l1 = 0.0;
        for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            double a = (double)avals[e];
            int64_t j = colidx[e];
            for (int32_t t = 0; t < k; ++t) {
                double term = a * xs_vals[j * k + t];
                int32_t c = xs_idx[j * k + t];
                h[c] += term;
                if (l1elem) l1elem[i * D + c] += fabs(term);
                row_l1 += fabs(term);
            }
        }
        if (l1row) l1row[i] = row_l1;
    }
}

/* ------------------------------------------------------------------------ */
/* Stable transpose (Alg. 2, stage 1: "transpose A to CSC").  Row j of the    */
/* result lists the entries of column j in increasing original row, and for   */
/* equal rows in original storage order.                                      */
/* ------------------------------------------------------------------------ */
void orc_csr_transpose(int64_t n_rows, int64_t n_cols, const int32_t* rowptr, const int32_t* colidx,
                       const float* vals, int32_t* t_rowptr, int32_t* t_colidx, float* t_vals) {
    for (int64_t j = 0; j <= n_cols; ++j) t_rowptr[j] = 0;
    for (int64_t p = 0; p < rowptr[n_rows]; ++p) t_rowptr[colidx[p] + 1] += 1;
    for (int64_t j = 0; j < n_cols; ++j) t_rowptr[j + 1] += t_rowptr[j];
    int32_t* cursor = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_cols > 0 ? n_cols : 1));
    for (int64_t j = 0; j < n_cols; ++j) cursor[j] = t_rowptr[j];
    for (int64_t i = 0; i < n_rows; ++i) {
        for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int32_t q = cursor[colidx[p]]++;
            t_colidx[q] = (int32_t)i;
            if (vals) t_vals[q] = vals[p];
        }
    }
    free(cursor);
}

/* ------------------------------------------------------------------------ */
/* DR-SpMM backward (Section 3.3: dL/dX = A^T dL/dY, evaluated only at the    */
/* CBSR indices preserved by the forward pass; Alg. 2 stage 2):               */
/*   G[j, t] = sum_{e in row j of A^T} a_e * dH[col_e, idx[j, t]]             */
/* At is given in CSR (N rows = sources, columns = destinations).             */
/* ------------------------------------------------------------------------ */
void orc_spmm_bwd(int64_t N, const int32_t* t_rowptr, const int32_t* t_colidx, const float* t_vals,
                  const double* dH, int32_t D, const int32_t* xs_idx, int32_t k,
                  double* G, double* l1elem, double* l1row) {
    for (int64_t j = 0; j < N; ++j) {
        double row_l1 = 0.0;
        for (int32_t t = 0; t < k; ++t) {
            int32_t c = xs_idx[j * k + t];
            double acc = 0.0, l1 = 0.0;
            for (int32_t e = t_rowptr[j]; e < t_rowptr[j + 1]; ++e) {
                double term = (double)t_vals[e] * dH[(int64_t)t_colidx[e] * D + c];
                acc += term;
                l1 += fabs(term);
            }
            G[j * k + t] = acc;
            if (l1elem) l1elem[j * k + t] = l1;
            row_l1 += l1;
        }
        if (l1row) l1row[j] = row_l1;
    }
}

/* ------------------------------------------------------------------------ */
/* Dense helpers for the module definitions (row vector times W convention,   */
/* as in the matrix form Y = A X W of Section 3.2).                           */
/* ------------------------------------------------------------------------ */

/* C[n, D] (+)= A[n, D] @ W[D, D] ;  L1[n, D] (+)= |A| @ |W| when L1 != NULL */
static void orc_matmul_acc(const double* A, const double* W, int64_t n, int32_t D, double* C, double* L1,
                           const double* Aabs) {
    for (int64_t i = 0; i < n; ++i)
        for (int32_t d = 0; d < D; ++d) {
            double a = A[i * D + d];
            double aa = Aabs ? Aabs[i * D + d] : fabs(a);
            if (a == 0.0 && aa == 0.0) continue;
            for (int32_t c = 0; c < D; ++c) {
                C[i * D + c] += a * W[d * D + c];
                if (L1) L1[i * D + c] += aa * fabs(W[d * D + c]);
            }
        }
}

/* C[n, D] = A[n, D] @ W^T */
static void orc_matmul_wt(const double* A, const double* W, int64_t n, int32_t D, double* C) {
    for (int64_t i = 0; i < n; ++i)
        for (int32_t d = 0; d < D; ++d) {
            double s = 0.0;
            for (int32_t c = 0; c < D; ++c) s += A[i * D + c] * W[d * D + c];
            C[i * D + d] = s;
        }
}

/* dW[D, D] = A^T[D, n] @ B[n, D] */
static void orc_matmul_at_b(const double* A, const double* B, int64_t n, int32_t D, double* dW) {
    for (int64_t q = 0; q < (int64_t)D * D; ++q) dW[q] = 0.0;
    for (int64_t i = 0; i < n; ++i)
        for (int32_t d = 0; d < D; ++d) {
            double a = A[i * D + d];
            if (a == 0.0) continue;
            for (int32_t c = 0; c < D; ++c) dW[d * D + c] += a * B[i * D + c];
        }
}

/* ------------------------------------------------------------------------ */
/* HeteroConv layer.  Relations (directions as in Section 2.2):               */
/*   near   cell->cell  SageConv(mean)   Z_near   = Xs_cell Wself_near + H_near  Wneigh_near   */
/*   pins   cell->net   SageConv(mean)   Y_net    = Xs_net  Wself_pins + H_pins  Wneigh_pins   */
/*   pinned net->cell   GraphConv(sym)   Z_pinned = H_pinned W_pinned                          */
/*   Y_cell = max(Z_near, Z_pinned), mask = [Z_near >= Z_pinned]  (Section 3.2 / 3.3)          */
/* with Xs_* = f(X_*), H_psi = A_psi f(X_src).  Aggregation first, projection second.          */
/* ------------------------------------------------------------------------ */

typedef struct {
    int64_t M, N;            /* destination rows, source columns */
    const int32_t* rowptr;   /* [M+1] */
    const int32_t* colidx;   /* [nnz] */
    const float* vals;       /* [nnz] */
} orc_csr;

typedef struct {
    const double* self_near;
    const double* neigh_near;
    const double* self_pins;
    const double* neigh_pins;
    const double* pinned;
} orc_weights;

/*
 * Forward.  Outputs (all caller-allocated):
 *   vals_cell[Nc,kc], idx_cell[Nc,kc], vals_net[Nn,kn], idx_net[Nn,kn]    CBSR of both node types
 *   H_near[Nc,D], H_pins[Nn,D], H_pinned[Nc,D]                            aggregated messages
 *   Z_near[Nc,D], Z_pinned[Nc,D]                                          module outputs at cell
 *   Y_cell[Nc,D], Y_net[Nn,D], mask[Nc,D] (1 = near branch won)
 *   l1_cell[Nc,D], l1_net[Nn,D]   sum of |contributing terms| per output element (bound on
 *                                 Z_near and Z_pinned jointly: the larger of the two L1 sums)
 */
int orc_heteroconv_fwd(int64_t Nc, int64_t Nn, int32_t D, int32_t kc, int32_t kn,
                       const orc_csr* near, const orc_csr* pins, const orc_csr* pinned,
                       const double* X_cell, const double* X_net, const orc_weights* W,
                       double* vals_cell, int32_t* idx_cell, double* vals_net, int32_t* idx_net,
                       double* H_near, double* H_pins, double* H_pinned,
                       double* Z_near, double* Z_pinned,
                       double* Y_cell, double* Y_net, uint8_t* mask,
                       double* l1_cell, double* l1_net) {
    if (near->M != Nc || near->N != Nc || pins->M != Nn || pins->N != Nc ||
        pinned->M != Nc || pinned->N != Nn) return -1;
    if (orc_topk(X_cell, Nc, D, kc, vals_cell, idx_cell)) return -1;
    if (orc_topk(X_net, Nn, D, kn, vals_net, idx_net)) return -1;

    size_t cd = (size_t)Nc * D, nd = (size_t)Nn * D;
    double* Xs_cell = (double*)malloc(sizeof(double) * cd);
    double* Xs_net = (double*)malloc(sizeof(double) * nd);
    double* habs = (double*)malloc(sizeof(double) * (cd > nd ? cd : nd));
    double* l1_pinned = (double*)malloc(sizeof(double) * cd);
    orc_densify(vals_cell, idx_cell, Nc, D, kc, Xs_cell);
    orc_densify(vals_net, idx_net, Nn, D, kn, Xs_net);

    /* near */
    orc_spmm_fwd(Nc, near->rowptr, near->colidx, near->vals, vals_cell, idx_cell, D, kc, H_near, habs, NULL);
    memset(Z_near, 0, sizeof(double) * cd);
    memset(l1_cell, 0, sizeof(double) * cd);
    orc_matmul_acc(Xs_cell, W->self_near, Nc, D, Z_near, l1_cell, NULL);
    orc_matmul_acc(H_near, W->neigh_near, Nc, D, Z_near, l1_cell, habs);

    /* pins */
    orc_spmm_fwd(Nn, pins->rowptr, pins->colidx, pins->vals, vals_cell, idx_cell, D, kc, H_pins, habs, NULL);
    memset(Y_net, 0, sizeof(double) * nd);
    memset(l1_net, 0, sizeof(double) * nd);
    orc_matmul_acc(Xs_net, W->self_pins, Nn, D, Y_net, l1_net, NULL);
    orc_matmul_acc(H_pins, W->neigh_pins, Nn, D, Y_net, l1_net, habs);

    /* pinned */
    orc_spmm_fwd(Nc, pinned->rowptr, pinned->colidx, pinned->vals, vals_net, idx_net, D, kn, H_pinned, habs, NULL);
    memset(Z_pinned, 0, sizeof(double) * cd);
    memset(l1_pinned, 0, sizeof(double) * cd);
    orc_matmul_acc(H_pinned, W->pinned, Nc, D, Z_pinned, l1_pinned, habs);

    /* merge at cell: element-wise max; ties go to the near branch */
    for (size_t q = 0; q < cd; ++q) {
        uint8_t m = (Z_near[q] >= Z_pinned[q]) ? 1 : 0;
        mask[q] = m;
        Y_cell[q] = m ? Z_near[q] : Z_pinned[q];
        if (l1_pinned[q] > l1_cell[q]) l1_cell[q] = l1_pinned[q];
    }
    free(Xs_cell); free(Xs_net); free(habs); free(l1_pinned);
    return 0;
}

/*
 * Backward, given what the forward saved (CBSR of both types, the three H, the mask).
 * Outputs: dX_cell[Nc,D], dX_net[Nn,D] (dense, zero outside the saved top-k positions),
 *          dXs_cell[Nc,kc], dXs_net[Nn,kn] (the same gradients in compact form),
 *          dW (five [D,D] matrices, order: self_near, neigh_near, self_pins, neigh_pins, pinned),
 *          l1_dxs_cell[Nc,kc], l1_dxs_net[Nn,kn]: sum of |terms| feeding each compact gradient
 *          (terms of the transposed SpMMs plus |self-term|).
 */
int orc_heteroconv_bwd(int64_t Nc, int64_t Nn, int32_t D, int32_t kc, int32_t kn,
                       const orc_csr* near, const orc_csr* pins, const orc_csr* pinned,
                       const orc_weights* W,
                       const double* vals_cell, const int32_t* idx_cell,
                       const double* vals_net, const int32_t* idx_net,
                       const double* H_near, const double* H_pins, const double* H_pinned,
                       const uint8_t* mask,
                       const double* dY_cell, const double* dY_net,
                       double* dX_cell, double* dX_net, double* dXs_cell, double* dXs_net,
                       double* dW_self_near, double* dW_neigh_near, double* dW_self_pins,
                       double* dW_neigh_pins, double* dW_pinned,
                       double* l1_dxs_cell, double* l1_dxs_net) {
    size_t cd = (size_t)Nc * D, nd = (size_t)Nn * D;
    double* dZ_near = (double*)malloc(sizeof(double) * cd);
    double* dZ_pinned = (double*)malloc(sizeof(double) * cd);
    double* dH = (double*)malloc(sizeof(double) * (cd > nd ? cd : nd));
    double* Xs = (double*)malloc(sizeof(double) * (cd > nd ? cd : nd));
    double* S = (double*)malloc(sizeof(double) * (cd > nd ? cd : nd));
    size_t gk = (size_t)Nc * kc > (size_t)Nn * kn ? (size_t)Nc * kc : (size_t)Nn * kn;
    double* G = (double*)malloc(sizeof(double) * gk);
    double* Gl1 = (double*)malloc(sizeof(double) * gk);

    /* route the cell gradient through the max-merge */
    for (size_t q = 0; q < cd; ++q) {
        dZ_near[q] = mask[q] ? dY_cell[q] : 0.0;
        dZ_pinned[q] = mask[q] ? 0.0 : dY_cell[q];
    }

    /* weight gradients */
    orc_densify(vals_cell, idx_cell, Nc, D, kc, Xs);
    orc_matmul_at_b(Xs, dZ_near, Nc, D, dW_self_near);
    orc_matmul_at_b(H_near, dZ_near, Nc, D, dW_neigh_near);
    orc_matmul_at_b(H_pinned, dZ_pinned, Nc, D, dW_pinned);
    orc_densify(vals_net, idx_net, Nn, D, kn, Xs);
    orc_matmul_at_b(Xs, dY_net, Nn, D, dW_self_pins);
    orc_matmul_at_b(H_pins, dY_net, Nn, D, dW_neigh_pins);

    /* transposed adjacencies */
    int32_t *nt_rp = (int32_t*)malloc(sizeof(int32_t) * (size_t)(Nc + 1));
    int32_t *pt_rp = (int32_t*)malloc(sizeof(int32_t) * (size_t)(Nc + 1));
    int32_t *qt_rp = (int32_t*)malloc(sizeof(int32_t) * (size_t)(Nn + 1));
    size_t e_near = (size_t)near->rowptr[near->M], e_pins = (size_t)pins->rowptr[pins->M],
           e_pinned = (size_t)pinned->rowptr[pinned->M];
    int32_t* nt_ci = (int32_t*)malloc(sizeof(int32_t) * (e_near + 1));
    int32_t* pt_ci = (int32_t*)malloc(sizeof(int32_t) * (e_pins + 1));
    int32_t* qt_ci = (int32_t*)malloc(sizeof(int32_t) * (e_pinned + 1));
    float* nt_v = (float*)malloc(sizeof(float) * (e_near + 1));
    float* pt_v = (float*)malloc(sizeof(float) * (e_pins + 1));
    float* qt_v = (float*)malloc(sizeof(float) * (e_pinned + 1));
    orc_csr_transpose(near->M, near->N, near->rowptr, near->colidx, near->vals, nt_rp, nt_ci, nt_v);
    orc_csr_transpose(pins->M, pins->N, pins->rowptr, pins->colidx, pins->vals, pt_rp, pt_ci, pt_v);
    orc_csr_transpose(pinned->M, pinned->N, pinned->rowptr, pinned->colidx, pinned->vals, qt_rp, qt_ci, qt_v);

    /* ---- cell sources: near^T and pins^T plus the near self term ---- */
    orc_matmul_wt(dZ_near, W->neigh_near, Nc, D, dH);                 /* dH_near */
    orc_spmm_bwd(Nc, nt_rp, nt_ci, nt_v, dH, D, idx_cell, kc, G, Gl1, NULL);
    for (size_t q = 0; q < (size_t)Nc * kc; ++q) { dXs_cell[q] = G[q]; l1_dxs_cell[q] = Gl1[q]; }
    orc_matmul_wt(dY_net, W->neigh_pins, Nn, D, dH);                  /* dH_pins */
    orc_spmm_bwd(Nc, pt_rp, pt_ci, pt_v, dH, D, idx_cell, kc, G, Gl1, NULL);
    for (size_t q = 0; q < (size_t)Nc * kc; ++q) { dXs_cell[q] += G[q]; l1_dxs_cell[q] += Gl1[q]; }
    orc_matmul_wt(dZ_near, W->self_near, Nc, D, S);                   /* self term, sampled */
    for (int64_t j = 0; j < Nc; ++j)
        for (int32_t t = 0; t < kc; ++t) {
            double s = S[j * D + idx_cell[j * kc + t]];
            dXs_cell[j * kc + t] += s;
            l1_dxs_cell[j * kc + t] += fabs(s);
        }

    /* ---- net sources: pinned^T plus the pins self term ---- */
    orc_matmul_wt(dZ_pinned, W->pinned, Nc, D, dH);                   /* dH_pinned */
    orc_spmm_bwd(Nn, qt_rp, qt_ci, qt_v, dH, D, idx_net, kn, G, Gl1, NULL);
    for (size_t q = 0; q < (size_t)Nn * kn; ++q) { dXs_net[q] = G[q]; l1_dxs_net[q] = Gl1[q]; }
    orc_matmul_wt(dY_net, W->self_pins, Nn, D, S);
    for (int64_t j = 0; j < Nn; ++j)
        for (int32_t t = 0; t < kn; ++t) {
            double s = S[j * D + idx_net[j * kn + t]];
            dXs_net[j * kn + t] += s;
            l1_dxs_net[j * kn + t] += fabs(s);
        }

    /* the top-k mask gates the whole gradient: scatter compact -> dense */
    memset(dX_cell, 0, sizeof(double) * cd);
    memset(dX_net, 0, sizeof(double) * nd);
    for (int64_t j = 0; j < Nc; ++j)
        for (int32_t t = 0; t < kc; ++t) dX_cell[j * D + idx_cell[j * kc + t]] = dXs_cell[j * kc + t];
    for (int64_t j = 0; j < Nn; ++j)
        for (int32_t t = 0; t < kn; ++t) dX_net[j * D + idx_net[j * kn + t]] = dXs_net[j * kn + t];

    free(dZ_near); free(dZ_pinned); free(dH); free(Xs); free(S); free(G); free(Gl1);
    free(nt_rp); free(pt_rp); free(qt_rp); free(nt_ci); free(pt_ci); free(qt_ci);
    free(nt_v); free(pt_v); free(qt_v);
    return 0;
}
