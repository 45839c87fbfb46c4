// Dense part of the HeteroConv layer (paper Section 3.2, matrix form Y = A X W, and its gradients in
// Section 3.3): the per-relation linear projections on the matrix cores, fp32 in and out
// (v_mfma_f32_32x32x2_f32), with the element-wise glue fused into the operand loads and epilogues:
//   - the D-ReLU output enters as CBSR and is densified on the fly into the LDS operand tile;
//   - the max-merge mask gates an operand while it is loaded (backward) or is produced by the
//     epilogue that merges the two cell branches (forward);
//   - the self-term gradient is sampled at the saved CBSR indices straight out of the accumulators.
#include "dr_internal.h"

namespace drc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kGemmThreads = 256;
constexpr int kBM = 128;   // rows per workgroup, 32 per wavefront
constexpr int kKC = 32;    // K chunk staged in LDS
constexpr int kAPad = 33;  // row stride of the A tile (bank-conflict-free column reads)

struct GemmParams {
    GemmOperand seg[2];
    int nseg;
    int rows;
    int D;
    int epi;
    float* out;
    uint8_t* mask_out;
    const uint16_t* sample_idx;
    int sample_k;
    float* compact;
};

// C tile element held by (lane, acc register r) of a 32x32 MFMA block
__device__ __forceinline__ int mfma_row(int lane, int r) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

template <int NT>  // NT = D / 32 column tiles
__global__ __launch_bounds__(kGemmThreads) void gemm_kernel(GemmParams p) {
    __shared__ float sA[kBM * kAPad];
    __shared__ float sB[kKC * (NT * 32 + 4)];
    constexpr int D = NT * 32;
    constexpr int kBStride = D + 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r0 = blockIdx.x * kBM;

    floatx16 acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;

    for (int sgi = 0; sgi < p.nseg; ++sgi) {
        const GemmOperand& sg = p.seg[sgi];
        for (int kk0 = 0; kk0 < D; kk0 += kKC) {
            // ---- A chunk [kBM x kKC] ----
            if (sg.dense) {
#pragma unroll
                for (int it = 0; it < (kBM * kKC / 4) / kGemmThreads; ++it) {
                    int q = it * kGemmThreads + tid;
                    int row = q >> 3, c4 = (q & 7) * 4;
                    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (r0 + row < p.rows) {
                        size_t off = (size_t)(r0 + row) * D + kk0 + c4;
                        v = *reinterpret_cast<const float4*>(sg.dense + off);
                        if (sg.mask) {
                            uchar4 m = *reinterpret_cast<const uchar4*>(sg.mask + off);
                            if (m.x != sg.mask_keep) v.x = 0.f;
                            if (m.y != sg.mask_keep) v.y = 0.f;
                            if (m.z != sg.mask_keep) v.z = 0.f;
                            if (m.w != sg.mask_keep) v.w = 0.f;
                        }
                    }
                    float* d = sA + row * kAPad + c4;
                    d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
                }
            } else {
                for (int q = tid; q < kBM * kAPad; q += kGemmThreads) sA[q] = 0.0f;
                __syncthreads();
                int row = tid & (kBM - 1);
                if (r0 + row < p.rows) {
                    const uint16_t* ri = sg.cbsr_idx + (size_t)(r0 + row) * sg.k;
                    const float* rv = sg.cbsr_vals + (size_t)(r0 + row) * sg.k;
                    for (int t = tid >> 7; t < sg.k; t += kGemmThreads / kBM) {
                        int c = ri[t];
                        if (c >= kk0 && c < kk0 + kKC) sA[row * kAPad + (c - kk0)] = rv[t];
                    }
                }
            }
            // ---- B chunk [kKC x D] ----
            if (!sg.transpose_w) {
#pragma unroll
                for (int it = 0; it < (kKC * D / 4) / kGemmThreads; ++it) {
                    int q = it * kGemmThreads + tid;
                    int kr = q / (D / 4), c4 = (q % (D / 4)) * 4;
                    float4 v = *reinterpret_cast<const float4*>(sg.W + (size_t)(kk0 + kr) * D + c4);
                    *reinterpret_cast<float4*>(sB + kr * kBStride + c4) = v;
                }
            } else {
                // B[kk][n] = W[n][kk0 + kk]
#pragma unroll
                for (int it = 0; it < (kKC * D / 4) / kGemmThreads; ++it) {
                    int q = it * kGemmThreads + tid;
                    int n = q >> 3, k4 = (q & 7) * 4;
                    float4 v = *reinterpret_cast<const float4*>(sg.W + (size_t)n * D + kk0 + k4);
                    sB[(k4 + 0) * kBStride + n] = v.x;
                    sB[(k4 + 1) * kBStride + n] = v.y;
                    sB[(k4 + 2) * kBStride + n] = v.z;
                    sB[(k4 + 3) * kBStride + n] = v.w;
                }
            }
            __syncthreads();
            // ---- multiply ----
            const float* arow = sA + (wave * 32 + (lane & 31)) * kAPad + (lane >> 5);
            const float* brow = sB + (lane >> 5) * kBStride + (lane & 31);
#pragma unroll
            for (int kk = 0; kk < kKC; kk += 2) {
                float a = arow[kk];
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    float b = brow[kk * kBStride + j * 32];
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[j], 0, 0, 0);
                }
            }
            __syncthreads();
        }
    }

    // ---- epilogue ----
    if (p.epi == kEpiStore || p.epi == kEpiMaxMerge) {
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int row = r0 + wave * 32 + mfma_row(lane, r);
                if (row < p.rows) {
                    size_t off = (size_t)row * D + j * 32 + (lane & 31);
                    float c = acc[j][r];
                    if (p.epi == kEpiMaxMerge) {
                        float prev = p.out[off];
                        bool near_wins = prev >= c;
                        p.mask_out[off] = near_wins ? 1 : 0;
                        c = near_wins ? prev : c;
                    }
                    p.out[off] = c;
                }
            }
    } else {
        // compact[row, t] += C[row, idx[row, t]] : stage one 32-column block at a time in sA
        const int row_l = tid & (kBM - 1);
        const int row_g = r0 + row_l;
        for (int j = 0; j < NT; ++j) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sA[(wave * 32 + mfma_row(lane, r)) * kAPad + (lane & 31)] = acc[j][r];
            __syncthreads();
            if (row_g < p.rows) {
                const uint16_t* ri = p.sample_idx + (size_t)row_g * p.sample_k;
                float* rc = p.compact + (size_t)row_g * p.sample_k;
                for (int t = tid >> 7; t < p.sample_k; t += kGemmThreads / kBM) {
                    int c = ri[t];
                    if ((c >> 5) == j) rc[t] += sA[row_l * kAPad + (c & 31)];
                }
            }
            __syncthreads();
        }
    }
}

int launch_gemm(const GemmOperand* segs, int nseg, int64_t rows, int D, GemmEpilogue epi, float* out,
                uint8_t* mask_out, const uint16_t* sample_idx, int sample_k, float* compact, hipStream_t s) {
    if (rows == 0) return DR_OK;
    GemmParams p{};
    for (int i = 0; i < nseg; ++i) p.seg[i] = segs[i];
    p.nseg = nseg;
    p.rows = (int)rows;
    p.D = D;
    p.epi = (int)epi;
    p.out = out;
    p.mask_out = mask_out;
    p.sample_idx = sample_idx;
    p.sample_k = sample_k;
    p.compact = compact;
    dim3 grid((unsigned)((rows + kBM - 1) / kBM)), block(kGemmThreads);
    switch (D / 32) {
        case 1: hipLaunchKernelGGL(gemm_kernel<1>, grid, block, 0, s, p); break;
        case 2: hipLaunchKernelGGL(gemm_kernel<2>, grid, block, 0, s, p); break;
        case 3: hipLaunchKernelGGL(gemm_kernel<3>, grid, block, 0, s, p); break;
        case 4: hipLaunchKernelGGL(gemm_kernel<4>, grid, block, 0, s, p); break;
        default: return fail(DR_ERR_UNSUPPORTED, "projection width D = %d not in {32,64,96,128}", D);
    }
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

// ---------------------------------------------------------------------------------------------------
// weight gradients  dW[D,D] = A^T B  (reduction over the graph's rows): each workgroup reduces a slab
// of rows into a full D x D accumulator held in MFMA registers and writes it to scratch; a second
// kernel sums the slabs in a fixed order (deterministic, no atomics).
// ---------------------------------------------------------------------------------------------------
constexpr int kWgRC = 32;  // rows staged per step

struct WgradParams {
    WgradOperand op;
    int rows;
    int rows_per_block;
    float* scratch;
};

template <int NT>
__global__ __launch_bounds__(kGemmThreads) void wgrad_partial_kernel(WgradParams p) {
    constexpr int D = NT * 32;
    constexpr int kStride = D + 4;
    __shared__ float sA[kWgRC * kStride];
    __shared__ float sB[kWgRC * kStride];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rb = blockIdx.x * p.rows_per_block;
    const int re = min(rb + p.rows_per_block, p.rows);

    // wavefront w owns output row-tiles w, w+4, ... ; all NT column tiles of each
    constexpr int kRT = (NT + 3) / 4;
    floatx16 acc[kRT][NT];
#pragma unroll
    for (int a = 0; a < kRT; ++a)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][j][r] = 0.0f;

    for (int rr = rb; rr < re; rr += kWgRC) {
        // stage B (and dense A) rows [rr, rr+32)
        for (int q = tid; q < kWgRC * D / 4; q += kGemmThreads) {
            int row = q / (D / 4), c4 = (q % (D / 4)) * 4;
            float4 vb = make_float4(0.f, 0.f, 0.f, 0.f), va = vb;
            if (rr + row < re) {
                size_t off = (size_t)(rr + row) * D + c4;
                vb = *reinterpret_cast<const float4*>(p.op.b + off);
                if (p.op.b_mask) {
                    uchar4 m = *reinterpret_cast<const uchar4*>(p.op.b_mask + off);
                    if (m.x != p.op.b_mask_keep) vb.x = 0.f;
                    if (m.y != p.op.b_mask_keep) vb.y = 0.f;
                    if (m.z != p.op.b_mask_keep) vb.z = 0.f;
                    if (m.w != p.op.b_mask_keep) vb.w = 0.f;
                }
                if (p.op.a_dense) va = *reinterpret_cast<const float4*>(p.op.a_dense + off);
            }
            *reinterpret_cast<float4*>(sB + row * kStride + c4) = vb;
            *reinterpret_cast<float4*>(sA + row * kStride + c4) = va;
        }
        if (!p.op.a_dense) {
            __syncthreads();
            for (int q = tid; q < kWgRC * p.op.k; q += kGemmThreads) {
                int row = q / p.op.k, t = q % p.op.k;
                if (rr + row < re) {
                    size_t off = (size_t)(rr + row) * p.op.k + t;
                    sA[row * kStride + p.op.a_cbsr_idx[off]] = p.op.a_cbsr_vals[off];
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < kWgRC; kk += 2) {
            const int r = kk + (lane >> 5);
            float b[NT];
#pragma unroll
            for (int j = 0; j < NT; ++j) b[j] = sB[r * kStride + j * 32 + (lane & 31)];
#pragma unroll
            for (int a = 0; a < kRT; ++a) {
                int dt = wave + 4 * a;
                if (dt < NT) {
                    float av = sA[r * kStride + dt * 32 + (lane & 31)];
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[a][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, b[j], acc[a][j], 0, 0, 0);
                }
            }
        }
        __syncthreads();
    }

    float* out = p.scratch + (size_t)blockIdx.x * D * D;
#pragma unroll
    for (int a = 0; a < kRT; ++a) {
        int dt = wave + 4 * a;
        if (dt < NT) {
#pragma unroll
            for (int j = 0; j < NT; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    out[(size_t)(dt * 32 + mfma_row(lane, r)) * D + j * 32 + (lane & 31)] = acc[a][j][r];
        }
    }
}

__global__ void wgrad_reduce_kernel(const float* __restrict__ scratch, int nb, int dd, float* __restrict__ dW) {
    int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= dd) return;
    float s = 0.0f;
    for (int b = 0; b < nb; ++b) s += scratch[(size_t)b * dd + q];
    dW[q] = s;
}

static int wgrad_blocks(int64_t rows) {
    int64_t nb = (rows + 1023) / 1024;
    if (nb > 1024) nb = 1024;
    if (nb < 1) nb = 1;
    return (int)nb;
}

size_t wgrad_scratch_bytes(int64_t rows, int D) { return sizeof(float) * (size_t)wgrad_blocks(rows) * D * D; }

int launch_wgrad(const WgradOperand& op, int64_t rows, int D, float* dW, void* scratch, hipStream_t s) {
    int nb = wgrad_blocks(rows);
    int rpb = (int)((rows + nb - 1) / nb);
    rpb = (rpb + kWgRC - 1) / kWgRC * kWgRC;
    if (rpb < kWgRC) rpb = kWgRC;
    nb = (int)((rows + rpb - 1) / rpb);
    if (nb < 1) nb = 1;
    WgradParams p{op, (int)rows, rpb, static_cast<float*>(scratch)};
    dim3 grid((unsigned)nb), block(kGemmThreads);
    switch (D / 32) {
        case 1: hipLaunchKernelGGL(wgrad_partial_kernel<1>, grid, block, 0, s, p); break;
        case 2: hipLaunchKernelGGL(wgrad_partial_kernel<2>, grid, block, 0, s, p); break;
        case 3: hipLaunchKernelGGL(wgrad_partial_kernel<3>, grid, block, 0, s, p); break;
        case 4: hipLaunchKernelGGL(wgrad_partial_kernel<4>, grid, block, 0, s, p); break;
        default: return fail(DR_ERR_UNSUPPORTED, "projection width D = %d not in {32,64,96,128}", D);
    }
    int dd = D * D;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((dd + 255) / 256), dim3(256), 0, s, static_cast<float*>(scratch),
                       nb, dd, dW);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

// ---------------------------------------------------------------------------------------------------
// compact gradient [n,k] -> dense [n,D], zero outside the saved top-k positions (the D-ReLU mask gates
// the whole gradient).  One wavefront per row, the row is assembled in LDS and stored coalesced.
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void scatter_compact_kernel(const float* __restrict__ compact,
                                                              const uint16_t* __restrict__ idx, int n, int D, int k,
                                                              float* __restrict__ dense) {
    extern __shared__ float srow[];  // [4][D]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float* row = srow + wave * D;
    const int waves = gridDim.x * 4;
    for (int i = blockIdx.x * 4 + wave; i < n; i += waves) {
        // LDS operations of one wavefront complete in issue order, so zero-fill, scatter and read-back
        // need no barrier between them; the wave barriers only pin the instruction order.
        for (int c = lane; c < D; c += kWave) row[c] = 0.0f;
        __builtin_amdgcn_wave_barrier();
        for (int t = lane; t < k; t += kWave) row[idx[(size_t)i * k + t]] = compact[(size_t)i * k + t];
        __builtin_amdgcn_wave_barrier();
        for (int c = lane; c < D; c += kWave) dense[(size_t)i * D + c] = row[c];
        __builtin_amdgcn_wave_barrier();
    }
}

int launch_scatter_compact(const float* compact, const uint16_t* idx, int64_t n, int D, int k, float* dense,
                           hipStream_t s) {
    if (n == 0) return DR_OK;
    long blocks = (n + 3) / 4;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(scatter_compact_kernel, dim3((unsigned)blocks), dim3(256), sizeof(float) * 4 * D, s, compact,
                       idx, (int)n, D, k, dense);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

}  // namespace drc
