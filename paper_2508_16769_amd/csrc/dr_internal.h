// Internal declarations shared by the HIP translation units of libdrcgnn (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstddef>
#include <cstdint>
#include <cstdio>

#include "dr_circuitgnn.h"

namespace drc {

constexpr int kWave = 64;      // CDNA wavefront width
constexpr int kNumXcd = 8;     // MI355X: 8 accelerator complex dies, one L2 each

// thread-local error text ------------------------------------------------------------------------
void set_error(const char* fmt, ...);
int fail(int code, const char* fmt, ...);
int hip_fail(hipError_t e, const char* what);

#define DRC_HIP(call)                                                   \
    do {                                                                \
        hipError_t drc_e__ = (call);                                    \
        if (drc_e__ != hipSuccess) return ::drc::hip_fail(drc_e__, #call); \
    } while (0)

#define DRC_REQUIRE(cond, ...)                                          \
    do {                                                                \
        if (!(cond)) return ::drc::fail(DR_ERR_INVALID_ARG, __VA_ARGS__); \
    } while (0)

#define DRC_TRY(expr)                  \
    do {                               \
        int drc_rc__ = (expr);         \
        if (drc_rc__) return drc_rc__; \
    } while (0)

int check_csr(const dr_csr* A, const char* name, bool need_vals);
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline hipStream_t as_stream(void* s) { return static_cast<hipStream_t>(s); }

// Workgroups are dealt to the XCDs round-robin by workgroup id.  Remap so that each XCD walks one
// contiguous range of logical tiles (neighbouring tiles share gathered rows in that XCD's L2).
// `per_xcd` = ceil(n_tiles / kNumXcd); launch per_xcd * kNumXcd workgroups and drop ids >= n_tiles.
__device__ __forceinline__ int xcd_contiguous_tile(int wg, int per_xcd) {
    return (wg % kNumXcd) * per_xcd + wg / kNumXcd;
}

// launchers (host side, argument checks already done by the ABI layer) ------------------------------
int launch_topk(const float* X, int64_t n, int D, int k, float* vals, uint16_t* idx, hipStream_t s);
// the same rows selected at two widths in one pass over X (vals2 == nullptr: only the first)
int launch_topk2(const float* X, int64_t n, int D, int k, float* vals, uint16_t* idx, int k2, float* vals2, uint16_t* idx2,
                 hipStream_t s);
int launch_spmm_fwd(const dr_csr* A, const float* xs_vals, const uint16_t* xs_idx, int D, int k, float* H,
                    hipStream_t s);
int launch_spmm_bwd(const dr_csr* At, const float* dH, const uint16_t* xs_idx, int D, int k, float* dXs,
                    int accumulate, hipStream_t s);
int launch_topk_ranked(const float* X, int64_t n, int D, int k, float* vals, uint16_t* idx, hipStream_t s);
int launch_spmm_fwd_adaptive(const dr_csr* A, const float* xr_vals, const uint16_t* xr_idx, int D, const dr_degree_classes* c,
                             float* H, hipStream_t s);
int launch_spmm_bwd_adaptive(const dr_csr* At, const uint8_t* edge_class, const float* dH, const uint16_t* xr_idx, int D,
                             const dr_degree_classes* c, float* dXr, int accumulate, hipStream_t s);
int launch_edge_classes(const dr_csr* At, const int32_t* a_rowptr, const dr_degree_classes* c, uint8_t* out, hipStream_t s);
int launch_csr_transpose(const dr_csr* A, int32_t* t_rowptr, int32_t* t_colidx, float* t_vals, void* ws,
                         hipStream_t s);
int launch_csr_normalize(int mode, int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t* rowptr,
                         const int32_t* colidx, float* vals_out, void* ws, hipStream_t s);
int launch_csr_normalize_noalloc(int mode, int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t* rowptr,
                                 const int32_t* colidx, float* vals_out, hipStream_t s);
int launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t s);
// DR-SpMM backward with the gathered rows staged in LDS, tile by tile (staged.hip)
int spmm_plan_create(dr_spmm_plan** out, const dr_csr* A, const int32_t* row_order, int D, hipStream_t s);
void spmm_plan_destroy(dr_spmm_plan* p);
int launch_spmm_bwd_planned(const dr_spmm_plan* p, const float* dH, const uint16_t* xs_idx, int k, float* dXs, int accumulate,
                            hipStream_t s);

// shape of a layer context (heteroconv.hip owns the struct)
struct HeteroDims {
    int64_t Nc, Nn;
    int D;
    int k_near, k_pins, k_self, k_pinned;   // D-ReLU widths: cells for near / for pins, nets for the pins self term / for pinned
};
HeteroDims heteroconv_dims(const dr_heteroconv* c);
const dr_csr* heteroconv_relations(const dr_heteroconv* c);
void heteroconv_capacity(const dr_heteroconv* c, int64_t* cells, int64_t* nets);   // what the context's buffers are sized for   // [3] near, pins, pinned as given to the create call
// A context whose buffers are sized for graphs of up to (Nc, Nn, E[near, pins, pinned]); relations are bound later
// (and again) with heteroconv_bind.  keep_workspace: also keep the transpose workspaces, which heteroconv_bind needs.
int heteroconv_create_capacity(dr_heteroconv** ctx, int64_t Nc, int64_t Nn, const int64_t E[3], int32_t D, int32_t k_near,
                               int32_t k_pins, int32_t k_self, int32_t k_pinned, bool keep_workspace);
int heteroconv_bind(dr_heteroconv* c, const dr_csr* near, const dr_csr* pins, const dr_csr* pinned, hipStream_t s);
// heteroconv_fwd / heteroconv_bwd with what a stacked model knows folded in (see ForwardOptions / BackwardOptions).
struct ForwardOptions {
    bool relu_out = false;          // clamp Y_cell and Y_net at zero as they are written (the mask compares raw values)
    bool skip_net_output = false;   // Y_net (and H_pins) are not wanted: the pins module is not evaluated
};
int heteroconv_forward(dr_heteroconv* c, const float* X_cell, const float* X_net, const dr_heteroconv_weights* W, float* Y_cell,
                       float* Y_net, const dr_heteroconv_saved* S, void* stream, ForwardOptions opt);
struct BackwardOptions {
    bool gate_inputs = false;     // zero dX where the layer's input was not positive (ReLU in front of the layer)
    bool skip_dx = false;         // weight gradients only: dX_cell / dX_net are not written (and may be null)
    bool dy_net_zero = false;     // dY_net is all zeros: what it would feed is not computed (fills instead)
};
int heteroconv_backward(dr_heteroconv* c, const float* dY_cell, const float* dY_net, const dr_heteroconv_weights* W,
                        const dr_heteroconv_saved* S, float* dX_cell, float* dX_net, const dr_heteroconv_wgrads* dW, void* stream,
                        BackwardOptions opt);
int heteroconv_create_widths(dr_heteroconv** ctx, const dr_csr* near, const dr_csr* pins, const dr_csr* pinned, int32_t D,
                             int32_t k_near, int32_t k_pins, int32_t k_self, int32_t k_pinned);

// dense part of the layer ------------------------------------------------------------------------------
struct GemmOperand {              // one K-segment of C = sum_seg A_seg * B_seg
    const float* dense;           // [rows, D] or nullptr
    const float* cbsr_vals;       // [rows, k] (with cbsr_idx) when the operand is a D-ReLU output
    const uint16_t* cbsr_idx;
    int k;
    const uint8_t* mask;          // optional [rows, D] gate applied to `dense`
    int mask_keep;                // keep elements whose mask byte equals this value
    const float* W;               // [D, D]
    int transpose_w;              // 0: B = W, 1: B = W^T
};
enum GemmEpilogue { kEpiStore = 0, kEpiMaxMerge = 1, kEpiSampleDense = 2 };
struct SampleSet {                // a top-k selection [rows, k] and a compact gradient that lives on it
    const uint16_t* idx;
    int k;
    const float* compact;         // [rows, k]; may be null in `first` (nothing to add to the sampled C)
    const float* gate;            // optional [rows, k]: the selected input values; out is zeroed where they are <= 0
};                                //   (the ReLU in front of the layer, applied to the layer's input gradient)
// C[rows, D] = sum over segments; epilogue:
//   kEpiStore       : out[rows,D] = C
//   kEpiMaxMerge    : mask_out = (out >= C); out = max(out, C)        (out holds the near branch on entry)
//   relu_out (kEpiStore, kEpiMaxMerge): what is written is clamped at zero (the mask still compares the raw values)
//   kEpiSampleDense : out[row,:] = 0, then out[row, first.idx[row,t]] = C[row, first.idx[row,t]] + first.compact[row,t],
//                     then (if second.idx) out[row, second.idx[row,t]] += second.compact[row,t]
int launch_gemm(const GemmOperand* segs, int nseg, int64_t rows, int D, GemmEpilogue epi, float* out,
                uint8_t* mask_out, SampleSet first, SampleSet second, hipStream_t s, int relu_out = 0);

struct WgradOperand {             // dW[D,D] = A^T B over `rows` rows
    const float* a_dense;         // [rows, D] or nullptr
    const float* a_cbsr_vals;     // CBSR alternative for A
    const uint16_t* a_cbsr_idx;
    int k;
    const float* b;               // [rows, D]
    const uint8_t* b_mask;        // optional gate on b
    int b_mask_keep;
};
size_t wgrad_scratch_bytes(int64_t rows, int D);
int launch_wgrad(const WgradOperand& op, int64_t rows, int D, float* dW, float* dW_cbsr, void* scratch, hipStream_t s);

}  // namespace drc
