// Dense part of the HeteroConv layer (paper Section 3.2, matrix form Y = A X W, and its gradients in
// Section 3.3): the per-relation linear projections on the matrix cores, fp32 in and out
// (v_mfma_f32_32x32x2_f32), with the element-wise glue fused into the operand loads and epilogues:
//   - the D-ReLU output enters as CBSR and is densified on the fly into the LDS operand tile;
//   - the max-merge mask gates an operand while it is loaded (backward) or is produced by the
//     epilogue that merges the two cell branches (forward);
//   - the self-term gradient is sampled at the saved CBSR indices straight out of the accumulators,
//     added to the compact SpMM gradient and written as the dense, top-k-gated dX rows.
//
// Projection kernel.  Persistent workgroups (a few per CU) loop over 64-row tiles.  The weights never
// touch LDS: wavefront w keeps the 32-column slab of W it is responsible for in registers in MFMA
// B-operand layout for the whole kernel (64 VGPRs per 128x128 weight), so the inner loop is one
// ds_read_b32 of the A operand per MFMA.  Row tiles are double-buffered through LDS: the global loads
// of the next tile are in flight while the current one is multiplied; one barrier per tile.
// These contractions run at the fp32 matrix rate (2*rows*D*D flops per weight); they are bound by the
// MFMA pipe, not by HBM, once the tiles stream (arithmetic intensity D/4 flop per byte moved).
#include "dr_internal.h"

#include <type_traits>

namespace drc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kPT = 256;  // threads per workgroup (4 wavefronts)

template <int NT> struct ProjCfg {
    static constexpr int D = 32 * NT;
    static constexpr int KS = D / 2;                                  // MFMA k-steps per segment
    static constexpr int RG = (NT >= 3) ? 1 : (NT == 2 ? 2 : 4);      // wavefront row groups
    static constexpr int BM = (NT == 1) ? 128 : 64;                   // rows per tile
    static constexpr int SPW = (BM / 32) / RG;                        // 32-row sub-tiles per wavefront
    static constexpr int LDA = D + 1;                                 // LDS row stride (conflict-free column reads)
    static constexpr int F4 = BM * D / 4 / kPT;                       // float4 per thread per dense tile
    static constexpr size_t kLds = sizeof(float) * 2 * BM * LDA;
};

struct GemmParams {
    GemmOperand seg[2];
    int nseg;
    int rows;
    int epi;
    float* out;
    uint8_t* mask_out;
    const uint16_t* sample_idx;
    int sample_k;
    const float* compact;
};

// C tile element held by (lane, acc register r) of a 32x32 MFMA block
__device__ __forceinline__ int mfma_row(int lane, int r) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

template <int NT, int NSEG>
__global__ __launch_bounds__(kPT, (NSEG == 1 ? 2 : 1)) void proj_kernel(GemmParams p) {
    using C = ProjCfg<NT>;
    constexpr int D = C::D, KS = C::KS, BM = C::BM, SPW = C::SPW, LDA = C::LDA, F4 = C::F4;
    extern __shared__ float smem[];
    float* const buf0 = smem;
    float* const buf1 = smem + BM * LDA;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ct = wave % NT, rg = wave / NT;
    const bool mm = rg < C::RG;                      // this wavefront multiplies (NT = 3 leaves one idle)
    const int n_tiles = (p.rows + BM - 1) / BM;
    if ((int)blockIdx.x >= n_tiles) return;

    // ---- weights of this wavefront's column slab, MFMA B-operand layout, resident in registers ----
    float breg[NSEG][KS];
#pragma unroll
    for (int sg = 0; sg < NSEG; ++sg) {
        const float* W = p.seg[sg].W;
        const bool tr = p.seg[sg].transpose_w != 0;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int kk = 2 * s + (lane >> 5), n = 32 * ct + (lane & 31);
            breg[sg][s] = mm ? (tr ? W[(size_t)n * D + kk] : W[(size_t)kk * D + n]) : 0.f;
        }
    }

    floatx16 acc[SPW];
#pragma unroll
    for (int j = 0; j < SPW; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;

    // Dense operand tile -> registers.  Only loads are issued here (the mask bytes ride along raw and are
    // applied when the tile is written to LDS), so the whole prefetch stays in flight during the multiply.
    float4 pre[F4];
    uint32_t prem[F4];
    auto prefetch = [&](int tile, int sg) {
        const GemmOperand& o = p.seg[sg];
        if (!o.dense) return;
#pragma unroll
        for (int it = 0; it < F4; ++it) {
            const int q = it * kPT + tid;
            const int row = q / (D / 4), c4 = (q % (D / 4)) * 4;
            const int grow = min(tile * BM + row, p.rows - 1);          // clamped: loads are unconditional
            const size_t off = (size_t)grow * D + c4;
            pre[it] = *reinterpret_cast<const float4*>(o.dense + off);
            prem[it] = o.mask ? *reinterpret_cast<const uint32_t*>(o.mask + off) : 0u;
        }
    };
    auto commit = [&](int tile, int sg, float* b) {  // registers (or CBSR rows) -> LDS tile
        const GemmOperand& o = p.seg[sg];
        if (o.dense) {
            const uint32_t keep = (uint32_t)o.mask_keep;
            const bool masked = o.mask != nullptr;
#pragma unroll
            for (int it = 0; it < F4; ++it) {
                const int q = it * kPT + tid;
                const int row = q / (D / 4), c4 = (q % (D / 4)) * 4;
                const bool in = tile * BM + row < p.rows;
                const uint32_t m = prem[it];
                float* d = b + row * LDA + c4;
                d[0] = (in && (!masked || ((m >> 0) & 0xffu) == keep)) ? pre[it].x : 0.f;
                d[1] = (in && (!masked || ((m >> 8) & 0xffu) == keep)) ? pre[it].y : 0.f;
                d[2] = (in && (!masked || ((m >> 16) & 0xffu) == keep)) ? pre[it].z : 0.f;
                d[3] = (in && (!masked || ((m >> 24) & 0xffu) == keep)) ? pre[it].w : 0.f;
            }
        } else {
            for (int q = tid; q < BM * LDA; q += kPT) b[q] = 0.0f;
            __syncthreads();
            const int k = o.k, total = BM * k;
            for (int q0 = 0; q0 < total; q0 += 8 * kPT) {      // 8 independent pair loads per thread, then the writes
                float v[8];
                int c[8], dst[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int q = q0 + u * kPT + tid;
                    const int row = q / k, t = q - row * k;
                    const int grow = tile * BM + row;
                    const bool ok = q < total && grow < p.rows;
                    const size_t off = ok ? (size_t)grow * k + t : 0;
                    v[u] = o.cbsr_vals[off];
                    c[u] = o.cbsr_idx[off];
                    dst[u] = ok ? row * LDA : -1;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (dst[u] >= 0) b[dst[u] + c[u]] = v[u];
            }
        }
    };
    // A operands are read from LDS two k-steps ahead of the MFMAs that consume them (explicit software
    // pipeline; the scheduling barriers keep the compiler from sinking the reads back next to their use).
    auto multiply = [&](const float* b, auto sg_tag) {
        constexpr int SG = decltype(sg_tag)::value;
        if (!mm) return;
        const float* a0 = b + ((rg * SPW) * 32 + (lane & 31)) * LDA + (lane >> 5);
        float a[3][SPW];
#pragma unroll
        for (int j = 0; j < SPW; ++j) { a[0][j] = a0[j * 32 * LDA]; a[1][j] = a0[j * 32 * LDA + 2]; }
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (s + 2 < KS) {
#pragma unroll
                for (int j = 0; j < SPW; ++j) a[(s + 2) % 3][j] = a0[j * 32 * LDA + 2 * (s + 2)];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < SPW; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s % 3][j], breg[SG][s], acc[j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    int tile = blockIdx.x, sg = 0, cur = 0;
    prefetch(tile, sg);
    commit(tile, sg, buf0);
    __syncthreads();
    for (;;) {
        int ntile = tile, nsg = sg + 1;
        if (nsg == NSEG) { nsg = 0; ntile = tile + gridDim.x; }
        const bool has_next = ntile < n_tiles;
        float* const bcur = cur ? buf1 : buf0;
        float* const bother = cur ? buf0 : buf1;
        if (has_next) prefetch(ntile, nsg);
        if (NSEG == 1 || sg == 0) multiply(bcur, std::integral_constant<int, 0>{});
        else multiply(bcur, std::integral_constant<int, NSEG - 1>{});

        if (sg == NSEG - 1) {
            // ---- epilogue of this row tile ----
            if (p.epi == kEpiStore) {
                if (mm) {
#pragma unroll
                    for (int j = 0; j < SPW; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int row = tile * BM + (rg * SPW + j) * 32 + mfma_row(lane, r);
                            if (row < p.rows) p.out[(size_t)row * D + 32 * ct + (lane & 31)] = acc[j][r];
                        }
                }
            } else if (p.epi == kEpiMaxMerge) {
                if (mm) {
#pragma unroll
                    for (int j = 0; j < SPW; ++j) {
                        float prev[16];
#pragma unroll
                        for (int r = 0; r < 16; ++r) {       // all loads of the other branch first (clamped rows)
                            const int row = min(tile * BM + (rg * SPW + j) * 32 + mfma_row(lane, r), p.rows - 1);
                            prev[r] = p.out[(size_t)row * D + 32 * ct + (lane & 31)];
                        }
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int row = tile * BM + (rg * SPW + j) * 32 + mfma_row(lane, r);
                            if (row < p.rows) {
                                const size_t off = (size_t)row * D + 32 * ct + (lane & 31);
                                const float c = acc[j][r];
                                const bool near_wins = prev[r] >= c;
                                p.mask_out[off] = near_wins ? 1 : 0;
                                if (!near_wins) p.out[off] = c;
                            }
                        }
                    }
                }
            } else {
                // out[row, :] = 0 except out[row, idx[row,t]] = compact[row,t] + C[row, idx[row,t]]
                if (mm) {
#pragma unroll
                    for (int j = 0; j < SPW; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            bother[((rg * SPW + j) * 32 + mfma_row(lane, r)) * LDA + 32 * ct + (lane & 31)] = acc[j][r];
                }
                __syncthreads();                                   // C tile complete; bcur no longer read
                for (int q = tid; q < BM * LDA; q += kPT) bcur[q] = 0.0f;
                __syncthreads();
                const int k = p.sample_k, total = BM * k;
                for (int q0 = 0; q0 < total; q0 += 8 * kPT) {
                    float v[8];
                    int c[8], dst[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int q = q0 + u * kPT + tid;
                        const int row = q / k, t = q - row * k;
                        const int grow = tile * BM + row;
                        const bool ok = q < total && grow < p.rows;
                        const size_t off = ok ? (size_t)grow * k + t : 0;
                        v[u] = p.compact[off];
                        c[u] = p.sample_idx[off];
                        dst[u] = ok ? row * LDA : -1;
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (dst[u] >= 0) bcur[dst[u] + c[u]] = v[u] + bother[dst[u] + c[u]];
                }
                __syncthreads();
                for (int q = tid; q < BM * D; q += kPT) {
                    const int row = q / D, c = q - row * D;
                    const int grow = tile * BM + row;
                    if (grow < p.rows) p.out[(size_t)grow * D + c] = bcur[row * LDA + c];
                }
                __syncthreads();
            }
#pragma unroll
            for (int j = 0; j < SPW; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
        }
        if (has_next) commit(ntile, nsg, bother);
        __syncthreads();
        if (!has_next) break;
        tile = ntile; sg = nsg; cur ^= 1;
    }
}

template <int NT, int NSEG>
static int launch_proj(const GemmParams& p, hipStream_t s) {
    using C = ProjCfg<NT>;
    static bool configured = false;
    if (!configured) {
        DRC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&proj_kernel<NT, NSEG>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::kLds));
        configured = true;
    }
    const int n_tiles = (p.rows + C::BM - 1) / C::BM;
    int grid = 512;                                    // about two resident workgroups per CU
    if (grid > n_tiles) grid = n_tiles;
    hipLaunchKernelGGL((proj_kernel<NT, NSEG>), dim3((unsigned)grid), dim3(kPT), C::kLds, s, p);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

int launch_gemm(const GemmOperand* segs, int nseg, int64_t rows, int D, GemmEpilogue epi, float* out,
                uint8_t* mask_out, const uint16_t* sample_idx, int sample_k, const float* compact, hipStream_t s) {
    if (rows == 0) return DR_OK;
    GemmParams p{};
    for (int i = 0; i < nseg; ++i) p.seg[i] = segs[i];
    p.nseg = nseg;
    p.rows = (int)rows;
    p.epi = (int)epi;
    p.out = out;
    p.mask_out = mask_out;
    p.sample_idx = sample_idx;
    p.sample_k = sample_k;
    p.compact = compact;
    const int key = (D / 32) * 10 + nseg;
    switch (key) {
        case 11: return launch_proj<1, 1>(p, s);
        case 12: return launch_proj<1, 2>(p, s);
        case 21: return launch_proj<2, 1>(p, s);
        case 22: return launch_proj<2, 2>(p, s);
        case 31: return launch_proj<3, 1>(p, s);
        case 32: return launch_proj<3, 2>(p, s);
        case 41: return launch_proj<4, 1>(p, s);
        case 42: return launch_proj<4, 2>(p, s);
        default: return fail(DR_ERR_UNSUPPORTED, "projection width D = %d not in {32,64,96,128}", D);
    }
}

// ---------------------------------------------------------------------------------------------------
// weight gradients  dW[D,D] = A^T B  (reduction over the graph's rows).  Persistent workgroups reduce a
// contiguous slab of rows each: 32-row chunks of A and B are double-buffered through LDS, the full
// D x D accumulator lives in MFMA registers (wavefront w owns row-tile w of dW), and the per-workgroup
// partials are summed by a second kernel in a fixed order (deterministic, no atomics).
// ---------------------------------------------------------------------------------------------------
constexpr int kWgRC = 32;  // rows staged per step

struct WgradParams {
    WgradOperand op;
    int rows;
    int rows_per_block;
    float* scratch;
};

template <int NT>
__global__ __launch_bounds__(kPT) void wgrad_partial_kernel(WgradParams p) {
    constexpr int D = NT * 32;
    constexpr int LD = D + 4;
    constexpr int F4 = kWgRC * D / 4 / kPT;      // float4 per thread per operand chunk (NT: 1..4)
    extern __shared__ float smem[];
    float* const sA0 = smem;
    float* const sB0 = sA0 + kWgRC * LD;
    float* const sA1 = sB0 + kWgRC * LD;
    float* const sB1 = sA1 + kWgRC * LD;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rb = blockIdx.x * p.rows_per_block;
    const int re = min(rb + p.rows_per_block, p.rows);
    const bool mm = wave < NT;                   // wavefront w owns dW rows [32w, 32w+32)

    floatx16 acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;

    // loads only (mask bytes raw); masking and range checks happen when the chunk is written to LDS
    float4 preA[F4], preB[F4];
    uint32_t prem[F4];
    auto prefetch = [&](int rr) {
#pragma unroll
        for (int it = 0; it < F4; ++it) {
            const int q = it * kPT + tid;
            const int row = q / (D / 4), c4 = (q % (D / 4)) * 4;
            const size_t off = (size_t)min(rr + row, re - 1) * D + c4;
            preB[it] = *reinterpret_cast<const float4*>(p.op.b + off);
            prem[it] = p.op.b_mask ? *reinterpret_cast<const uint32_t*>(p.op.b_mask + off) : 0u;
            preA[it] = p.op.a_dense ? *reinterpret_cast<const float4*>(p.op.a_dense + off)
                                    : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto commit = [&](int rr, float* sA, float* sB) {
        const uint32_t keep = (uint32_t)p.op.b_mask_keep;
        const bool masked = p.op.b_mask != nullptr;
#pragma unroll
        for (int it = 0; it < F4; ++it) {
            const int q = it * kPT + tid;
            const int row = q / (D / 4), c4 = (q % (D / 4)) * 4;
            const bool in = rr + row < re;
            const uint32_t m = prem[it];
            float4 vb, va;
            vb.x = (in && (!masked || ((m >> 0) & 0xffu) == keep)) ? preB[it].x : 0.f;
            vb.y = (in && (!masked || ((m >> 8) & 0xffu) == keep)) ? preB[it].y : 0.f;
            vb.z = (in && (!masked || ((m >> 16) & 0xffu) == keep)) ? preB[it].z : 0.f;
            vb.w = (in && (!masked || ((m >> 24) & 0xffu) == keep)) ? preB[it].w : 0.f;
            va = in ? preA[it] : make_float4(0.f, 0.f, 0.f, 0.f);           // zeros when A is CBSR
            *reinterpret_cast<float4*>(sB + row * LD + c4) = vb;
            *reinterpret_cast<float4*>(sA + row * LD + c4) = va;
        }
        if (!p.op.a_dense) {
            __syncthreads();
            const int k = p.op.k, total = kWgRC * k;
            for (int q0 = 0; q0 < total; q0 += 4 * kPT) {
                float v[4];
                int c[4], dst[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int q = q0 + u * kPT + tid;
                    const int row = q / k, t = q - row * k;
                    const bool ok = q < total && rr + row < re;
                    const size_t off = ok ? (size_t)(rr + row) * k + t : 0;
                    v[u] = p.op.a_cbsr_vals[off];
                    c[u] = p.op.a_cbsr_idx[off];
                    dst[u] = ok ? row * LD : -1;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (dst[u] >= 0) sA[dst[u] + c[u]] = v[u];
            }
        }
    };

    if (rb < re) {
        int cur = 0;
        prefetch(rb);
        commit(rb, sA0, sB0);
        __syncthreads();
        for (int rr = rb; rr < re; rr += kWgRC) {
            const bool has_next = rr + kWgRC < re;
            const float* sA = cur ? sA1 : sA0;
            const float* sB = cur ? sB1 : sB0;
            if (has_next) prefetch(rr + kWgRC);
            if (mm) {
                // operands of k-step i+1 are read from LDS before the MFMAs of k-step i are issued
                const float* pa = sA + (lane >> 5) * LD + wave * 32 + (lane & 31);
                const float* pb = sB + (lane >> 5) * LD + (lane & 31);
                float av[2], b[2][NT];
                av[0] = pa[0];
#pragma unroll
                for (int j = 0; j < NT; ++j) b[0][j] = pb[j * 32];
#pragma unroll
                for (int i = 0; i < kWgRC / 2; ++i) {
                    if (i + 1 < kWgRC / 2) {
                        av[(i + 1) & 1] = pa[(2 * i + 2) * LD];
#pragma unroll
                        for (int j = 0; j < NT; ++j) b[(i + 1) & 1][j] = pb[(2 * i + 2) * LD + j * 32];
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i & 1], b[i & 1][j], acc[j], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (has_next) commit(rr + kWgRC, cur ? sA0 : sA1, cur ? sB0 : sB1);
            __syncthreads();
            cur ^= 1;
        }
    }

    float* out = p.scratch + (size_t)blockIdx.x * D * D;
    if (mm) {
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                out[(size_t)(wave * 32 + mfma_row(lane, r)) * D + j * 32 + (lane & 31)] = acc[j][r];
    }
}

// dW[q] = sum over partials, fixed order: wavefront j of a workgroup sums every 8th partial starting at j
// for 64 consecutive outputs, then the 8 wavefront sums are added in order.
__global__ __launch_bounds__(512) void wgrad_reduce_kernel(const float* __restrict__ scratch, int nb, int dd,
                                                           float* __restrict__ dW) {
    __shared__ float part[8][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = blockIdx.x * 64 + lane;
    float s = 0.0f;
    if (q < dd)
        for (int b = wave; b < nb; b += 8) s += scratch[(size_t)b * dd + q];
    part[wave][lane] = s;
    __syncthreads();
    if (wave == 0 && q < dd) {
        float t = 0.0f;
#pragma unroll
        for (int w = 0; w < 8; ++w) t += part[w][lane];
        dW[q] = t;
    }
}

static int wgrad_blocks(int64_t rows) {
    int64_t nb = (rows + kWgRC - 1) / kWgRC;
    if (nb > 512) nb = 512;
    if (nb < 1) nb = 1;
    return (int)nb;
}

size_t wgrad_scratch_bytes(int64_t rows, int D) { return sizeof(float) * (size_t)wgrad_blocks(rows) * D * D; }

template <int NT>
static int launch_wgrad_nt(const WgradParams& p, int nb, hipStream_t s) {
    constexpr size_t lds = sizeof(float) * 4 * kWgRC * (NT * 32 + 4);
    static bool configured = false;
    if (!configured) {
        DRC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_partial_kernel<NT>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        configured = true;
    }
    hipLaunchKernelGGL(wgrad_partial_kernel<NT>, dim3((unsigned)nb), dim3(kPT), lds, s, p);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

int launch_wgrad(const WgradOperand& op, int64_t rows, int D, float* dW, void* scratch, hipStream_t s) {
    int nb = wgrad_blocks(rows);
    int rpb = (int)((rows + nb - 1) / nb);
    rpb = (rpb + kWgRC - 1) / kWgRC * kWgRC;
    if (rpb < kWgRC) rpb = kWgRC;
    nb = (int)((rows + rpb - 1) / rpb);
    if (nb < 1) nb = 1;
    WgradParams p{op, (int)rows, rpb, static_cast<float*>(scratch)};
    int rc;
    switch (D / 32) {
        case 1: rc = launch_wgrad_nt<1>(p, nb, s); break;
        case 2: rc = launch_wgrad_nt<2>(p, nb, s); break;
        case 3: rc = launch_wgrad_nt<3>(p, nb, s); break;
        case 4: rc = launch_wgrad_nt<4>(p, nb, s); break;
        default: return fail(DR_ERR_UNSUPPORTED, "projection width D = %d not in {32,64,96,128}", D);
    }
    if (rc) return rc;
    const int dd = D * D;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((dd + 63) / 64)), dim3(512), 0, s,
                       static_cast<float*>(scratch), nb, dd, dW);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

}  // namespace drc
