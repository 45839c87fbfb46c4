/*
 * dr_circuitgnn.h -- C ABI of the MI355X (gfx950) implementation of the DR-CircuitGNN
 * HeteroConv hot path: row-wise Dynamic-ReLU (top-k) of the node embeddings, the DR-SpMM of
 * each relation's CSR adjacency with the resulting row-sparse operand, and the backward SpMM
 * on the transposed adjacency evaluated at the saved top-k positions.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Plain C.  No exceptions cross the boundary.  Every call returns an int status:
 *    DR_OK (0) or a negative DR_ERR_* code; dr_last_error() returns a thread-local message.
 *  - Every array argument is a caller-owned DEVICE pointer (HBM of the current HIP device),
 *    borrowed until the enqueued work has finished.  dr_csr structs themselves live on the
 *    host; the three pointers inside them are device pointers.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *    enqueue work; none of them synchronises the host.
 *  - All arguments are validated on the host before anything is launched, so argument
 *    errors are reported without touching the GPU.
 *  - Matrices are row-major fp32; graph indices are int32; CBSR column indices are uint16.
 *  - Relations are stored as CSR with rows = destination nodes and columns = source nodes
 *    (the paper's A^psi, M_dst x N_src).  Column order inside a row is free and duplicate
 *    entries are allowed; they count as separate edges.
 *  - CBSR (compressed balanced sparse row, paper Section 3.1): for each embedding row exactly k
 *    (value, column) pairs, stored as vals[n,k] and idx[n,k] with columns ascending.
 */
#ifndef DR_CIRCUITGNN_H
#define DR_CIRCUITGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DR_OK               0
#define DR_ERR_INVALID_ARG (-1)  /* null pointer, k < 1, k > D, bad shape, misaligned pointer, ... */
#define DR_ERR_UNSUPPORTED (-2)  /* legal request outside what this build implements (e.g. D too large) */
#define DR_ERR_HIP         (-3)  /* a HIP runtime call failed; message carries hipGetErrorString */
#define DR_ERR_WORKSPACE   (-4)  /* workspace_bytes smaller than the matching *_workspace_bytes() */

#define DR_NORM_MEAN 0           /* SageConv 'mean' aggregation: a_ij = 1 / deg_in(i)                       */
#define DR_NORM_SYM  1           /* GraphConv: a_ij = 1 / sqrt(max(deg_in(i),1) * max(deg_out(j),1))        */

#define DR_MAX_D 1024            /* largest embedding width accepted by dr_topk / dr_spmm_*                 */

/* CSR adjacency of one relation.  rowptr[n_rows+1], colidx[nnz], vals[nnz] are device pointers.
 * vals may be NULL only where a call says so.  nnz must be < 2^31 and equal rowptr[n_rows]. */
typedef struct dr_csr {
    int64_t n_rows;          /* M: destination nodes */
    int64_t n_cols;          /* N: source nodes      */
    int64_t nnz;             /* E: stored edges      */
    const int32_t* rowptr;
    const int32_t* colidx;
    const float* vals;
} dr_csr;

/* Message of the last failing call on this thread ("" if none). */
const char* dr_last_error(void);

/* ABI version of this header (bumped on incompatible change). */
int dr_abi_version(void);

/*
 * (1) D-ReLU, paper Section 3.1 (threshold th_i = min(topk(X_i, k)) and the piecewise f(X)).
 * For each of the n rows of X[n,D] keep exactly the k largest signed values (no clamping of
 * negatives); among equal values the lower column wins; -0.0 and +0.0 compare equal.  Writes the
 * survivors in ascending column order: vals[n,k] (bit copies of the inputs) and idx[n,k].
 * Precondition: inputs finite.  Requires 1 <= k <= D <= DR_MAX_D.  n == 0 is a no-op.
 */
int dr_topk(const float* X, int64_t n, int32_t D, int32_t k,
            float* vals, uint16_t* idx, void* stream);

/*
 * (2) DR-SpMM forward, paper Section 3.2 / Alg. 1:  H[M,D] = A * f(X), with f(X) given as the CBSR
 * (xs_vals[N,k], xs_idx[N,k]) of the source node type:
 *     H[i,c] = sum over edges e of row i, pairs t:  A.vals[e] * xs_vals[colidx[e], t]  where xs_idx[colidx[e], t] == c.
 * H is fully overwritten; rows without edges become zeros.  fp32 accumulation, order unspecified.
 * Requires A->vals != NULL, 1 <= k <= D <= DR_MAX_D, every xs_idx < D (not checked).
 */
int dr_spmm_fwd(const dr_csr* A, const float* xs_vals, const uint16_t* xs_idx,
                int32_t D, int32_t k, float* H, void* stream);

/*
 * (3) DR-SpMM backward, paper Section 3.3 / Alg. 2: gradient w.r.t. the k surviving entries of every
 * source row, using the transposed adjacency At (CSR of A^T: N rows = sources, M columns =
 * destinations), the dense upstream gradient dH[M,D] and the CBSR indices saved by the forward:
 *     dXs[j,t] (=|+=) sum over edges e of row j of At:  At.vals[e] * dH[At.colidx[e], xs_idx[j,t]].
 * accumulate == 0 overwrites dXs[N,k]; accumulate != 0 adds to its current contents (the paper's
 * accumulation of the per-relation pieces, done without atomics on HBM).
 */
int dr_spmm_bwd(const dr_csr* At, const float* dH, const uint16_t* xs_idx,
                int32_t D, int32_t k, float* dXs, int accumulate, void* stream);

/*
 * DR-SpMM backward with the gathered rows staged in LDS (paper Section 3.3 / Alg. 2 stage 2, which keeps the interim
 * rows of a block in shared memory).  Same result as dr_spmm_bwd, for relations in which nearby rows share most of
 * their neighbours (the geometric `near` relation).  A plan is made once per transposed relation:
 *   row_order: device array of At->n_rows row ids, a permutation -- the order in which the rows are processed; runs
 *              of up to 64 consecutive entries form the tiles whose distinct dH rows are loaded into LDS once.  NULL =
 *              the rows' own order.  The order changes no result (every sum keeps its storage order); it pays when
 *              rows that share neighbours sit next to each other, e.g. cells sorted along a space-filling curve of
 *              their placement.
 * dr_spmm_plan_create reads At on the host (it waits for `stream`), allocates the plan's device arrays and returns
 * DR_ERR_UNSUPPORTED when D is not a multiple of 32, when a single row does not fit a tile (more than 2048 edges, or
 * more distinct neighbours than 64 KB / (4 * min(D, 64)) rows) or when the device offers too little LDS; the caller
 * then stays with dr_spmm_bwd.  dr_spmm_plan_info reports the number of tiles and `reuse` = stored edges per distinct
 * gathered row summed over the tiles (the factor by which the dH rows fetched per edge shrink).  At, its arrays and
 * row_order are not referenced after dr_spmm_plan_create returns.
 * dr_spmm_bwd_planned: arguments as dr_spmm_bwd (D is the plan's); dH must be 16-byte aligned; k <= min(D, 2 * min(D, 64)).
 */
typedef struct dr_spmm_plan dr_spmm_plan;
int dr_spmm_plan_create(dr_spmm_plan** plan, const dr_csr* At, const int32_t* row_order, int32_t D, void* stream);
int dr_spmm_plan_info(const dr_spmm_plan* plan, int64_t* n_tiles, double* reuse);
int dr_spmm_bwd_planned(const dr_spmm_plan* plan, const float* dH, const uint16_t* xs_idx, int32_t k, float* dXs,
                        int accumulate, void* stream);
int dr_spmm_plan_destroy(dr_spmm_plan* plan);

/*
 * Degree-adaptive K (paper Section 3.2, Alg. 1 stage 2 "dynamic warp partitioning" and the text after Alg. 1):
 * neighbour groups are classified by their size, and the larger a destination's neighbour group the fewer entries
 * of each neighbour's embedding it receives (K1 > K2 > K3).  The paper prints no formula, boundaries or K values;
 * this build takes them as arguments and defines, for a relation with CSR A (rows = destinations):
 *     K(i) = k1 if deg(i) <= t1,  k2 if t1 < deg(i) <= t2,  k3 otherwise          (deg = stored entries of row i of A)
 *     H[i,:] = sum over edges (i <- j):  A.vals[e] * f_{K(i)}(X_j)                 (f_K: the K largest entries of the row)
 * and the backward as the derivative of that with the selections held fixed.  The row-sparse operand is stored in
 * RANK order -- pair t of a row is its t-th largest value (ties: lower column first) -- so every f_K with K <= k1
 * is a prefix of the k1 stored pairs.
 */
typedef struct dr_degree_classes {
    int32_t t1, t2;        /* 0 <= t1 <= t2 */
    int32_t k1, k2, k3;    /* min(D, 64) >= k1 >= k2 >= k3 >= 1 */
} dr_degree_classes;

/* D-ReLU in rank order: vals[n,k], idx[n,k] hold the k largest signed values of every row of X[n,D], largest first
 * (same selection and tie rule as dr_topk; only the order of the pairs differs).  Requires 1 <= k <= D <= DR_MAX_D. */
int dr_topk_ranked(const float* X, int64_t n, int32_t D, int32_t k, float* vals, uint16_t* idx, void* stream);

/* Forward: H[M,D] fully overwritten.  (xr_vals, xr_idx): rank-ordered CBSR [N, cls->k1] of the source node type. */
int dr_spmm_fwd_adaptive(const dr_csr* A, const float* xr_vals, const uint16_t* xr_idx, int32_t D,
                         const dr_degree_classes* cls, float* H, void* stream);

/* Setup for the backward: the degree class (0 low, 1 medium, 2 high) of the destination of every stored entry of
 * At = CSR of A^T, read from A's own row pointers A_rowptr[M+1] (device).  edge_class[At->nnz], one byte each.
 * Only t1 and t2 of cls are used. */
int dr_degree_edge_classes(const dr_csr* At, const int32_t* A_rowptr, const dr_degree_classes* cls, uint8_t* edge_class,
                           void* stream);

/* Backward: dXr[j,t] (=|+=) sum over edges e of row j of At with t < K(class of e):
 *     At.vals[e] * dH[At.colidx[e], xr_idx[j,t]],        dXr[N, cls->k1] in the rank order of xr_idx.
 * edge_class: what dr_degree_edge_classes wrote for the same At and boundaries (values above 2 are not checked).
 * Requires M < 2^30. */
int dr_spmm_bwd_adaptive(const dr_csr* At, const uint8_t* edge_class, const float* dH, const uint16_t* xr_idx, int32_t D,
                         const dr_degree_classes* cls, float* dXr, int accumulate, void* stream);

/*
 * Setup: stable CSR transpose (Alg. 2 stage 1, "transpose A to CSC").  Row j of the result lists the
 * entries of column j of A in increasing original row and, for equal rows, original storage order.
 * Outputs t_rowptr[n_cols+1], t_colidx[nnz], t_vals[nnz] (t_vals and A->vals may both be NULL for a
 * pattern-only transpose).  Integer-exact and deterministic.  Every A->colidx must lie in [0, n_cols) and rowptr must
 * be non-decreasing with rowptr[n_rows] == nnz (device data, not checked).  workspace: device scratch of at least
 * dr_csr_transpose_workspace_bytes() bytes, 256-byte aligned, contents undefined before and after.
 */
size_t dr_csr_transpose_workspace_bytes(int64_t n_rows, int64_t n_cols, int64_t nnz);
int dr_csr_transpose(const dr_csr* A, int32_t* t_rowptr, int32_t* t_colidx, float* t_vals,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * Setup: edge values of the three modules (GraphSAGE 'mean' mode and GCN normalisation, paper
 * Section 4.1): fills vals_out[nnz] for the pattern (rowptr, colidx) according to `mode`
 * (DR_NORM_MEAN or DR_NORM_SYM).  Values are evaluated in fp64 and rounded once to fp32.
 * workspace: at least dr_csr_normalize_workspace_bytes() bytes (0 for DR_NORM_MEAN; may be NULL then).
 */
size_t dr_csr_normalize_workspace_bytes(int mode, int64_t n_rows, int64_t n_cols, int64_t nnz);
int dr_csr_normalize(int mode, int64_t n_rows, int64_t n_cols, int64_t nnz,
                     const int32_t* rowptr, const int32_t* colidx, float* vals_out,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * dr_csr_normalize for callers that cannot allocate device memory or bring a workspace (code under HIP graph
 * capture, serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same results bit
 * for bit.  The column counts of DR_NORM_SYM live in an array of DR_NOALLOC_MAX_COLS + 1 int32 (8 MiB) that is part of
 * the library image on every GPU it runs on; the call allocates and frees nothing.  n_cols above DR_NOALLOC_MAX_COLS
 * is refused with DR_ERR_UNSUPPORTED (DR_NORM_MEAN needs no scratch and has no such limit).  All calls on one GPU
 * share that array: calls that overlap on one GPU (different streams, different threads) race and must be
 * serialised by the caller.
 */
#define DR_NOALLOC_MAX_COLS (1 << 21)
int dr_csr_normalize_noalloc(int mode, int64_t n_rows, int64_t n_cols, int64_t nnz,
                             const int32_t* rowptr, const int32_t* colidx, float* vals_out, void* stream);

/* ------------------------------------------------------------------------------------------------
 * The HeteroConv layer (paper Fig. 3, Sections 3.2-3.4): three relation modules on three HIP streams,
 *     near   (cell->cell, SageConv mean):  Z_near   = f(X_cell) Wself_near + (A_near   f(X_cell)) Wneigh_near
 *     pins   (cell->net,  SageConv mean):  Y_net    = f(X_net)  Wself_pins + (A_pins   f(X_cell)) Wneigh_pins
 *     pinned (net->cell,  GraphConv sym):  Z_pinned =                        (A_pinned f(X_net))  W_pinned
 *     Y_cell = max(Z_near, Z_pinned) element-wise, mask = [Z_near >= Z_pinned]   (ties go to near)
 * and the matching backward (gradient routed by mask, transposed SpMM gated by the saved indices).
 * Every weight is [D,D] row-major with the Y = X W convention; there are no biases.
 * ---------------------------------------------------------------------------------------------- */

typedef struct dr_heteroconv dr_heteroconv;   /* opaque: transposed adjacencies, streams, events, scratch */

typedef struct dr_heteroconv_weights {        /* device pointers, each [D,D]; read-only in fwd and bwd */
    const float* self_near;
    const float* neigh_near;
    const float* self_pins;
    const float* neigh_pins;
    const float* pinned;
} dr_heteroconv_weights;

typedef struct dr_heteroconv_wgrads {         /* device pointers, each [D,D]; overwritten by heteroconv_bwd */
    float* self_near;
    float* neigh_near;
    float* self_pins;
    float* neigh_pins;
    float* pinned;
} dr_heteroconv_wgrads;

typedef struct dr_heteroconv_saved {          /* caller-owned device buffers written by fwd, read by bwd */
    float*    vals_cell;  /* [Nc,k_cell] CBSR of the cell embeddings (k_near with one K per relation)  */
    uint16_t* idx_cell;   /* [Nc,k_cell]                                                               */
    float*    vals_net;   /* [Nn,k_net]  CBSR of the net embeddings (k_pinned with one K per relation) */
    uint16_t* idx_net;    /* [Nn,k_net]                                                                */
    float*    H_near;     /* [Nc,D] aggregated messages per relation  */
    float*    H_pins;     /* [Nn,D]                                   */
    float*    H_pinned;   /* [Nc,D]                                   */
    uint8_t*  mask;       /* [Nc,D] 1 where the near branch won the max-merge */
    /* Only for contexts of heteroconv_create_per_relation; ignored (may be NULL) where the widths coincide: */
    float*    vals_cell_pins;  /* [Nc,k_pins] CBSR of the cells as the pins module reads them, if k_pins != k_near   */
    uint16_t* idx_cell_pins;   /* [Nc,k_pins]                                                                         */
    float*    vals_net_self;   /* [Nn,k_pins] CBSR of the nets as the pins self term reads them, if k_pins != k_pinned */
    uint16_t* idx_net_self;    /* [Nn,k_pins]                                                                         */
} dr_heteroconv_saved;

/*
 * Build the per-graph context: validates the three relations (near Nc x Nc, pins Nn x Nc,
 * pinned Nc x Nn, all with vals), transposes them on the device, creates three streams and the events
 * that join them, and allocates the scratch the backward pass needs.  Device memory is allocated only by the
 * *_create calls (released by the matching *_destroy) and, temporarily, by heteroconv_profile_k.  The CSR arrays passed in stay
 * owned by the caller and must outlive the context.  The call synchronises the device before returning.
 * Requires D in {32, 64, 96, 128}, 1 <= k_cell, k_net <= D.
 */
int heteroconv_create(dr_heteroconv** ctx, const dr_csr* near, const dr_csr* pins, const dr_csr* pinned,
                      int32_t D, int32_t k_cell, int32_t k_net);

/*
 * The same context with one K per edge type (paper Section 4.3: graph-specific k_near, k_pins, k_pinned).  D-ReLU
 * belongs to the module that reads the embedding, so every input of a module is sparsified with that module's K:
 *     Z_near   = f_{k_near}(X_cell) Wself_near + (A_near   f_{k_near}(X_cell))  Wneigh_near
 *     Y_net    = f_{k_pins}(X_net)  Wself_pins + (A_pins   f_{k_pins}(X_cell))  Wneigh_pins
 *     Z_pinned =                                 (A_pinned f_{k_pinned}(X_net)) W_pinned
 * A node type read with two different K gets two CBSRs (the extra buffers of dr_heteroconv_saved); in the backward
 * every use sends its gradient through its own selection and the pieces add up in the dense dX.
 * heteroconv_get_k reports the four widths a context uses: cells for near, cells for pins, nets for the pins self
 * term, nets for pinned (k_cell, k_cell, k_net, k_net for heteroconv_create).
 */
int heteroconv_create_per_relation(dr_heteroconv** ctx, const dr_csr* near, const dr_csr* pins, const dr_csr* pinned,
                                   int32_t D, int32_t k_near, int32_t k_pins, int32_t k_pinned);
int heteroconv_get_k(const dr_heteroconv* ctx, int32_t* k_near, int32_t* k_pins, int32_t* k_self, int32_t* k_pinned);

/*
 * Preprocessing: optimal-K profiling of one sub-graph (paper Sections 4.1 and 4.3: the DR-SpMM kernels are timed on
 * each sub-graph for K in {2, 4, ..., 64} and the fastest K of each edge type is used for training).  For every
 * relation (0 near, 1 pins, 2 pinned) and every candidate K the source embeddings go through D-ReLU at that K,
 * then dr_spmm_fwd and dr_spmm_bwd of the relation run `warmup` untimed and `reps` timed times (HIP events on
 * one stream).  X_cell[Nc,D], X_net[Nn,D]: representative embeddings on the device; they also stand in for the
 * upstream gradients of the backward (kernel time does not depend on the values).
 * ms_fwd, ms_bwd: HOST arrays [3 * n_candidates], relation-major, mean milliseconds per launch.
 * best_k: HOST array [3], for each relation the candidate with the least ms_fwd + ms_bwd (ties: the smaller K) --
 * the argument triple of heteroconv_create_per_relation.  The context only lends its transposed adjacencies and
 * D; the K it was created with plays no part.  Allocates and frees its own device scratch; synchronises the device.
 * Requires 1 <= candidates[i] <= D, 1 <= n_candidates <= 64, warmup >= 0, 1 <= reps <= 1000.
 */
int heteroconv_profile_k(dr_heteroconv* ctx, const float* X_cell, const float* X_net,
                         const int32_t* candidates, int32_t n_candidates, int32_t warmup, int32_t reps,
                         float* ms_fwd, float* ms_bwd, int32_t* best_k);

/*
 * Forward of one layer.  Inputs X_cell[Nc,D], X_net[Nn,D]; outputs Y_cell[Nc,D], Y_net[Nn,D] and every
 * buffer of `saved`.  Work is forked from `stream` onto the context's three relation streams and joined
 * back into `stream` before the call returns (device-side joins; the host does not wait).
 */
int heteroconv_fwd(dr_heteroconv* ctx, const float* X_cell, const float* X_net,
                   const dr_heteroconv_weights* W, float* Y_cell, float* Y_net,
                   const dr_heteroconv_saved* saved, void* stream);

/*
 * Backward of one layer.  Inputs dY_cell[Nc,D], dY_net[Nn,D], the weights and what fwd saved.  Outputs
 * dX_cell[Nc,D] and dX_net[Nn,D] (dense; exactly zero outside the saved top-k positions) and the five
 * weight gradients.  Same stream semantics as heteroconv_fwd.
 */
int heteroconv_bwd(dr_heteroconv* ctx, const float* dY_cell, const float* dY_net,
                   const dr_heteroconv_weights* W, const dr_heteroconv_saved* saved,
                   float* dX_cell, float* dX_net, const dr_heteroconv_wgrads* dW, void* stream);

/* Transposed adjacency of a relation held by the context (which: 0 near, 1 pins, 2 pinned); the
 * returned struct's pointers are device memory owned by the context. */
int heteroconv_get_transpose(const dr_heteroconv* ctx, int which, dr_csr* out);

int heteroconv_destroy(dr_heteroconv* ctx);

/*
 * Processing-order hint for the geometric `near` relation (paper Section 2.2: near links come from the cells'
 * placement).  cell_order: device array of Nc cell ids, a permutation, in which cells that lie close to each other in
 * the layout sit next to each other (e.g. sorted along a Z-order curve of their coordinates); NULL = the cells' own
 * order.  The layer's backward then runs the transposed `near` DR-SpMM through dr_spmm_plan / dr_spmm_bwd_planned (dH
 * rows of a tile of cells staged in LDS) -- provided the plan can be made and reuses a staged row at least twice on
 * average; *staged (may be NULL) reports whether it will.  No result changes with the order.  Builds the plan on the
 * host (waits for `stream` and for the context's transposes); call it once per bound graph, outside the timed loop.
 * A later re-binding of the context drops the plan.
 */
int heteroconv_set_cell_order(dr_heteroconv* ctx, const int32_t* cell_order, int* staged, void* stream);

/*
 * Relation concurrency (paper Section 3.4).  DR_OVERLAP_ON: the near, pins and pinned pipelines are enqueued on
 * three HIP streams and joined by events only where the data flow demands it.  DR_OVERLAP_OFF: the same kernels,
 * in the same dependency order, back to back on one stream.  DR_OVERLAP_AUTO (default): separate streams while one
 * relation's launches leave CUs idle at their tails (max(Nc, Nn) * D < 2^26), one stream beyond that, where
 * overlapping launches only time-slice the CUs.  Takes effect from the next heteroconv_fwd / heteroconv_bwd.
 */
#define DR_OVERLAP_AUTO 0
#define DR_OVERLAP_ON   1
#define DR_OVERLAP_OFF  2
int heteroconv_set_overlap(dr_heteroconv* ctx, int mode);

/*
 * Measurement aid (not part of the method): per-kernel device time of the layer's launches.
 * heteroconv_profile(ctx, 1) makes every later heteroconv_fwd / heteroconv_bwd bracket each of its kernel
 * launches with a pair of HIP events recorded on the stream that launch runs on; heteroconv_profile(ctx, 0)
 * stops that.  heteroconv_kernel_times synchronises the device, adds up the elapsed time per kernel id since
 * the previous call into ms_sum[n] / launches[n] (host arrays, n >= heteroconv_num_kernels()) and forgets the
 * recorded launches.  heteroconv_kernel_name(id) names a kernel id ("dr_spmm_fwd.near", ...).
 * With profiling on, the calls create HIP events on demand (host-side allocation).
 */
int heteroconv_profile(dr_heteroconv* ctx, int enable);
int heteroconv_num_kernels(void);
const char* heteroconv_kernel_name(int id);
int heteroconv_kernel_times(dr_heteroconv* ctx, double* ms_sum, int64_t* launches, int n);

/* ------------------------------------------------------------------------------------------------
 * Multi-layer training step (paper Section 4.1: stacked HeteroConv layers with ReLU between them, a
 * per-cell congestion read-out, mean-squared error, Adam with weight decay), over a batch of independent
 * sub-graphs that share the parameters and are processed concurrently on HIP streams (Section 3.4).
 *
 *   X^(0) = input;  (Y_cell, Y_net) = HeteroConv_l(X^(l-1));  X^(l) = ReLU(Y) for l < L,  X^(L) = Y;
 *   pred_i = X_cell^(L)[i,:] . w_head;   loss = mean over all cells of the batch of (pred_i - target_i)^2.
 *
 * Parameters: one flat device vector theta of hgnn_num_params(L, D) = L*5*D*D + D floats,
 *   [layer 1: self_near, neigh_near, self_pins, neigh_pins, pinned (each [D,D] row-major) | layer 2 | ... | w_head[D]].
 * ---------------------------------------------------------------------------------------------- */

typedef struct dr_hgnn dr_hgnn;               /* opaque: activations, saved state and gradients of every sub-graph */

typedef struct dr_hgnn_layer_buffers {        /* device pointers owned by the model, for inspection */
    const float* X_cell;                      /* [Nc,D] input of the layer (caller's X for layer 0)              */
    const float* X_net;                       /* [Nn,D]                                                          */
    const float* Y_cell;                      /* [Nc,D] output of the layer, after ReLU unless it is the last    */
    const float* Y_net;                       /* [Nn,D]; NULL (like saved.H_pins) for the last layer without inspection */
    dr_heteroconv_saved saved;                /* what the layer's forward saved                                  */
    const float* dY_cell;                     /* [Nc,D] gradient that entered the layer's backward               */
    const float* dY_net;                      /* [Nn,D]                                                          */
    const float* dX_cell;                     /* [Nc,D] gradient the layer's backward produced; for layers > 0   */
    const float* dX_net;                      /* [Nn,D] already gated by the ReLU in front of the layer; NULL    */
                                              /* for layer 0 unless hgnn_set_inspection(model, 1) was called     */
    dr_heteroconv_wgrads dW;                  /* this sub-graph's share of the layer's weight gradients          */
} dr_hgnn_layer_buffers;

int64_t hgnn_num_params(int32_t n_layers, int32_t D);

/*
 * Build the model state for n_graphs sub-graphs (one heteroconv context each, all with the same D; every
 * sub-graph keeps the K its context was created with, per node type or per relation) and n_layers layers:
 * allocates every activation, saved-state and gradient buffer and one stream per sub-graph.  The contexts stay
 * owned by the caller and must outlive the model.  Synchronises the device.
 * Buffers are sized for what the contexts can hold, and every step works on the graphs bound to them at that
 * moment: over the contexts of dr_pipeline slots one model trains on a stream of sub-graphs.
 */
int hgnn_create(dr_hgnn** model, int32_t n_graphs, dr_heteroconv* const* graphs, int32_t n_layers);

/*
 * The same model with the batch stacked into ONE block-diagonal graph on the device (sub-graph q's rows and
 * columns shifted by the node counts of the sub-graphs before it): a step then issues one launch per kernel for the
 * whole batch instead of one per sub-graph, which is the faster mapping for small sub-graphs (a 20 000-cell launch
 * fills a fraction of the GPU).  The result is the same step: same selections, loss and gradient up to the order of
 * the fp32 sums over rows.  All contexts must have the same D and the same K; they only lend their relations and may
 * be destroyed once the call returns (the CSR arrays are copied).  hgnn_train_step takes the same per-sub-graph
 * pointer tables; inputs that already lie behind one another in memory (X_cell[q+1] == X_cell[q] + Nc_q * D, ...) are
 * read in place, others are first copied into a staging buffer.  hgnn_get_layer_buffers returns sub-graph q's rows
 * of the stacked buffers; dW is then the gradient of the whole batch for every q.
 */
int hgnn_create_batched(dr_hgnn** model, int32_t n_graphs, dr_heteroconv* const* graphs, int32_t n_layers);

/*
 * One training step.  X_cell[g] / X_net[g] / target[g]: host arrays of n_graphs device pointers
 * ([Nc_g,D], [Nn_g,D], [Nc_g]).  theta, adam_m, adam_v: device vectors of hgnn_num_params floats, updated in
 * place (step = 1 for the first update; moments start at zero); the hyper-parameters are doubles so that
 * 1 - beta and the bias corrections are formed exactly before they are rounded to the fp32 the kernel uses.  grad_out: device vector of the same
 * length that receives the batch gradient (before weight decay).  loss_out: one device float.
 * Work is forked from `stream` onto one stream per sub-graph (and the relation streams below them) and
 * joined back before the parameter update; the host never waits.
 */
int hgnn_train_step(dr_hgnn* model, const float* const* X_cell, const float* const* X_net,
                    const float* const* target, float* theta, float* adam_m, float* adam_v,
                    double lr, double beta1, double beta2, double eps, double weight_decay, int32_t step,
                    float* grad_out, float* loss_out, void* stream);

/* A training step does not need everything a layer can compute: the gradient of the input features is read by
 * nobody, so the first layer's backward computes its weight gradients only (no dH projections, transposed SpMMs or
 * dX write-outs); the read-out uses the cells only, so the last layer does not evaluate its pins module (no H_pins,
 * no Y_net), and its backward replaces what the all-zero dY_net would feed by fills.  Loss, gradient and update are
 * the same bits either way.  enable != 0 makes later steps compute those parts as well, for inspection through
 * hgnn_get_layer_buffers (which reports NULL for them otherwise). */
int hgnn_set_inspection(dr_hgnn* model, int enable);

/* Buffers of sub-graph `graph`, layer `layer` (valid after a step).  pred / dpred: [Nc] of that sub-graph
 * (layer argument ignored), may be NULL. */
int hgnn_get_layer_buffers(const dr_hgnn* model, int32_t graph, int32_t layer, dr_hgnn_layer_buffers* out,
                           const float** pred, const float** dpred);

int hgnn_destroy(dr_hgnn* model);

/* ------------------------------------------------------------------------------------------------
 * Host-side pipeline (paper Section 3.4 and the breakdown of Section 4.4: loading, initialisation and host-to-device
 * copies of the next sub-graphs run on CPU threads and their own streams while the GPU works on the current ones).
 * A pipeline owns n_slots slots; each has pinned staging memory, device arrays and a layer context sized for the
 * largest graph it will see (the capacities given at creation) and one stream.  Nothing is allocated after
 * dr_pipeline_create.  Per slot the calls go submit -> acquire -> (use the context) -> release -> submit ...
 * ---------------------------------------------------------------------------------------------- */

typedef struct dr_pipeline dr_pipeline;

typedef struct dr_host_graph {      /* HOST arrays (pageable or pinned), borrowed until dr_pipeline_acquire returns */
    int64_t n_cells, n_nets;
    int64_t nnz_near, nnz_pins;
    const int32_t* near_rowptr;     /* [n_cells+1]  rows = destination cells, columns = source cells */
    const int32_t* near_colidx;     /* [nnz_near]                                                    */
    const int32_t* pins_rowptr;     /* [n_nets+1]   rows = nets, columns = cells; pinned is its transpose pattern */
    const int32_t* pins_colidx;     /* [nnz_pins]                                                    */
    const float*   X_cell;          /* [n_cells,D] embeddings to upload with the graph, or NULL      */
    const float*   X_net;           /* [n_nets,D]  or NULL                                           */
} dr_host_graph;

/* Allocates the slots (device arrays, pinned staging, contexts with one K per node type) and starts n_threads
 * worker threads.  Synchronises the device. */
int dr_pipeline_create(dr_pipeline** pipeline, int32_t n_slots, int32_t n_threads, int64_t max_cells, int64_t max_nets,
                       int64_t max_nnz_near, int64_t max_nnz_pins, int32_t D, int32_t k_cell, int32_t k_net);

/* Hands a host graph to the worker threads and returns at once.  A worker waits (on the host) until the GPU has
 * finished with the slot's previous graph, stages the arrays in pinned memory and enqueues on the slot's stream:
 * the uploads, the pinned pattern (transpose of pins), the edge values of the three modules (dr_csr_normalize) and
 * the transposed adjacencies of the slot's context.  The slot must be idle (never used, or released). */
int dr_pipeline_submit(dr_pipeline* pipeline, int32_t slot, const dr_host_graph* graph);

/* Waits (host) until the slot's work has been ENQUEUED -- not until the GPU has done it -- and makes `stream` wait
 * for it on the device.  *ctx: the slot's layer context, bound to the submitted graph, for heteroconv_fwd / bwd,
 * hgnn_* or heteroconv_profile_k on `stream`.  *X_cell / *X_net (may be NULL): device copies of the uploaded
 * embeddings, or NULL where none were given.  A failure of the worker is reported here. */
int dr_pipeline_acquire(dr_pipeline* pipeline, int32_t slot, void* stream, dr_heteroconv** ctx,
                        const float** X_cell, const float** X_net);

/* The three relations (device CSRs with edge values) of an acquired slot: out[0] near, out[1] pins, out[2] pinned. */
int dr_pipeline_relations(dr_pipeline* pipeline, int32_t slot, dr_csr* out);

/* Marks the slot reusable once everything enqueued on `stream` so far has finished (an event; the host does not
 * wait).  The context and the device arrays of the slot must not be used by calls made after this one. */
int dr_pipeline_release(dr_pipeline* pipeline, int32_t slot, void* stream);

/* Stops the workers (queued submissions are still processed), waits for the device and frees everything. */
int dr_pipeline_destroy(dr_pipeline* pipeline);

#ifdef __cplusplus
}
#endif
#endif /* DR_CIRCUITGNN_H */
