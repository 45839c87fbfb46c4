// Dense part of the HeteroConv layer (paper Section 3.2, matrix form Y = A X W, and its gradients in
// Section 3.3): the per-relation linear projections on the matrix cores, fp32 in and out
// (v_mfma_f32_32x32x2_f32), with the element-wise glue fused into the operand loads and epilogues:
//   - the D-ReLU output enters as CBSR and is densified on the fly into the LDS operand tile;
//   - the max-merge mask gates an operand while it is loaded (backward) or is produced by the
//     epilogue that merges the two cell branches (forward);
//   - the self-term gradient is sampled at the saved CBSR indices straight out of the accumulators,
//     added to the compact SpMM gradient and written as the dense, top-k-gated dX rows.
//
// Projection kernel.  Persistent workgroups (as many as fit the chip at once: two to four per CU) loop over
// 32-row tiles (D >= 96; 64 or 128 rows for narrower D).  The weights never
// touch LDS: wavefront w keeps the 32-column slab of W it is responsible for in registers in MFMA
// B-operand layout for the whole kernel (64 VGPRs per 128x128 weight), so the inner loop is one
// ds_read_b128 of the A operand per four MFMAs.  Row tiles are double-buffered through LDS: every global
// load a tile needs (operand rows, mask bytes, CBSR pairs, the other branch for the max-merge) is issued
// before the multiply of the previous tile and consumed after it.  The operand kind and the epilogue are
// template parameters: with a single code path per instantiation every load has exactly one consumer, so
// the compiler's wait counters are placed at the consumers and not, conservatively, in front of the
// multiply.
// These contractions run at the fp32 matrix rate (2*rows*D*D flops per weight); they are bound by the
// MFMA pipe, not by HBM, once the tiles stream (arithmetic intensity D/4 flop per byte moved).
#include "dr_internal.h"

#include <atomic>
#include <type_traits>

namespace drc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kPT = 256;  // threads per workgroup (4 wavefronts)
constexpr int kCP = 8;    // CBSR pairs per thread that are prefetched into registers

enum AKind { kADense = 0, kADenseMasked = 1, kACbsrDense = 2 };   // last: segment 0 CBSR, segment 1 dense

template <int NT> struct ProjCfg {
    static constexpr int D = 32 * NT;
    static constexpr int KS = D / 2;                                  // MFMA k-steps per segment
    static constexpr int RG = (NT >= 3) ? 1 : (NT == 2 ? 2 : 4);      // wavefront row groups
    static constexpr int BM = (NT == 1) ? 128 : (NT == 2 ? 64 : 32);  // rows per tile
    static constexpr int SPW = (BM / 32) / RG;                        // 32-row sub-tiles per wavefront
    static constexpr int LDA = D + 4;                                 // LDS row stride: rows stay 16-byte aligned
    static constexpr int F4 = BM * D / 4 / kPT;                       // float4 per thread per dense tile
    static constexpr int TPR = kPT / BM;                              // threads that share one tile row
    static constexpr int RPW = BM / 4;                                // tile rows staged by one wavefront
    static constexpr size_t kLds = sizeof(float) * 2 * BM * LDA;
};

struct GemmParams {
    GemmOperand seg[2];
    int nseg;
    int rows;
    int epi;
    float* out;
    uint8_t* mask_out;
    SampleSet first, second;      // kEpiSampleDense(2): selections and compact gradients of the write-out
    int relu;                     // kEpiStore / kEpiMaxMerge: clamp what is written at zero
};
constexpr int kEpiSampleDense2 = 3;   // kEpiSampleDense with a second selection and/or no compact on the first

struct PairRegs {
    float v[kCP];
    uint32_t c[kCP];
};

// C tile element held by (lane, acc register r) of a 32x32 MFMA block
__device__ __forceinline__ int mfma_row(int lane, int r) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// Contraction index served by MFMA k-step s in lane half h.  Eight consecutive k form a group: half 0
// takes the first four, half 1 the last four, so a lane fetches the A values of four k-steps with one
// 16-byte LDS read.  The B registers are loaded in the same order.
__device__ __forceinline__ int mfma_k(int s, int h) { return 8 * (s >> 2) + 4 * h + (s & 3); }

// 16-byte load that does not displace cached lines (the four scalar loads merge into one instruction)
__device__ __forceinline__ float4 nt_load4(const float* p) {
    float4 v;
    v.x = __builtin_nontemporal_load(p);
    v.y = __builtin_nontemporal_load(p + 1);
    v.z = __builtin_nontemporal_load(p + 2);
    v.w = __builtin_nontemporal_load(p + 3);
    return v;
}


template <int NT, int AK, int EPI>
// wavefronts per SIMD the register budget is set for: 4 for the one-operand store kernels, 3 with the merge or
// sampling epilogue (they hold the other branch / the pairs as well), 2 with two resident weight slabs
__global__ __launch_bounds__(kPT, (EPI == kEpiStore ? (AK == kACbsrDense ? 2 : 4) : 3)) void proj_kernel(GemmParams p) {
    constexpr bool kSample2 = (EPI == kEpiSampleDense2);
    using C = ProjCfg<NT>;
    constexpr int D = C::D, KS = C::KS, BM = C::BM, SPW = C::SPW, LDA = C::LDA, F4 = C::F4;
    constexpr int TPR = C::TPR, RPW = C::RPW;
    constexpr int NSEG = (AK == kACbsrDense) ? 2 : 1;
    constexpr bool kMasked = (AK == kADenseMasked);
    extern __shared__ __align__(16) float smem[];
    float* const buf0 = smem;
    float* const buf1 = smem + BM * LDA;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ct = wave % NT, rg = wave / NT;
    const bool mm = rg < C::RG;                      // this wavefront multiplies (NT = 3 leaves one idle)
    const int prow = tid / TPR, ppart = tid % TPR;   // row-owned stagings: tile row and share of it
    const int n_tiles = (p.rows + BM - 1) / BM;
    if ((int)blockIdx.x >= n_tiles) return;

    // ---- weights of this wavefront's column slab, MFMA B-operand layout, resident in registers ----
    float breg[NSEG][KS];
#pragma unroll
    for (int sg = 0; sg < NSEG; ++sg) {
        // B[kk][n] = W[kk][n], or W[n][kk] for the transposed use: one strided load per element, no branches
        const int sk = p.seg[sg].transpose_w ? 1 : D, sn = p.seg[sg].transpose_w ? D : 1;
        const float* W = p.seg[sg].W + (32 * ct + (lane & 31)) * sn;
#pragma unroll
        for (int s = 0; s < KS; ++s) breg[sg][s] = W[mfma_k(s, lane >> 5) * sk];
    }

    floatx16 acc[SPW];
#pragma unroll
    for (int j = 0; j < SPW; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;

    // ---- dense operand tile: global -> registers -> LDS.  Wavefront w stages tile rows
    // [w*RPW, (w+1)*RPW); loads are unconditional on clamped rows, masks ride along raw. ----
    const GemmOperand& od = p.seg[NSEG - 1];
    float4 pre[F4];
    uint32_t prem[F4];
    auto prefetch = [&](int tile) {
#pragma unroll
        for (int it = 0; it < F4; ++it) {
            const int q = it * kWave + lane;
            const int row = wave * RPW + q / (D / 4), c4 = (q % (D / 4)) * 4;
            const size_t off = (size_t)min(tile * BM + row, p.rows - 1) * D + c4;
            pre[it] = nt_load4(od.dense + off);                         // operand rows are read once: streamed
            if (kMasked) prem[it] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(od.mask + off));
        }
    };
    auto commit = [&](int tile, float* b) {
        const uint32_t keep = (uint32_t)od.mask_keep;
#pragma unroll
        for (int it = 0; it < F4; ++it) {
            const int q = it * kWave + lane;
            const int row = wave * RPW + q / (D / 4), c4 = (q % (D / 4)) * 4;
            const bool in = tile * BM + row < p.rows;
            float4 v = pre[it];
            if (kMasked) {
                const uint32_t m = prem[it];
                v.x = (((m >> 0) & 0xffu) == keep) ? v.x : 0.f;
                v.y = (((m >> 8) & 0xffu) == keep) ? v.y : 0.f;
                v.z = (((m >> 16) & 0xffu) == keep) ? v.z : 0.f;
                v.w = (((m >> 24) & 0xffu) == keep) ? v.w : 0.f;
            }
            if (!in) v = make_float4(0.f, 0.f, 0.f, 0.f);
            *reinterpret_cast<float4*>(b + row * LDA + c4) = v;
        }
    };

    // ---- CBSR pairs of a tile, row-owned: thread (prow, ppart) holds pairs ppart, ppart+TPR, ... of tile
    // row prow.  The first kCP pairs per thread travel through registers; the rest (k > kCP*TPR) are
    // fetched when they are placed. ----
    auto load_pairs = [&](PairRegs& pr, const float* vals, const uint16_t* idx, int k, int tile) {
        const size_t base = (size_t)min(tile * BM + prow, p.rows - 1) * k;
#pragma unroll
        for (int u = 0; u < kCP; ++u) {
            const int t = min(ppart + TPR * u, k - 1);
            pr.v[u] = vals[base + t];
            pr.c[u] = idx[base + t];
        }
    };
    auto load_cols = [&](PairRegs& pr, const uint16_t* idx, int k, int tile) {       // columns only, values zero
        const size_t base = (size_t)min(tile * BM + prow, p.rows - 1) * k;
#pragma unroll
        for (int u = 0; u < kCP; ++u) {
            pr.v[u] = 0.f;
            pr.c[u] = idx[base + min(ppart + TPR * u, k - 1)];
        }
    };
    auto zero_own_part = [&](float* rowp) {
        const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int i = 0; i < D / TPR / 4; ++i) *reinterpret_cast<float4*>(rowp + ppart * (D / TPR) + 4 * i) = z;
        // The threads of one row sit in one wavefront and LDS executes a wavefront's accesses in order, so
        // the scattered writes that follow land on the zeroed row without a workgroup barrier.
        __builtin_amdgcn_wave_barrier();
    };
    // D-ReLU rows -> dense LDS tile.  Every write is unconditional: pairs past k go to the padding column,
    // rows past the end write zeros.
    auto stage_cbsr = [&](const PairRegs& pr, int tile, float* b) {
        const GemmOperand& o = p.seg[0];
        float* rowp = b + prow * LDA;
        zero_own_part(rowp);
        const int k = o.k;
        const bool rin = tile * BM + prow < p.rows;
#pragma unroll
        for (int u = 0; u < kCP; ++u) {
            const int t = ppart + TPR * u;
            rowp[t < k ? (int)pr.c[u] : D] = rin ? pr.v[u] : 0.f;
        }
        const size_t base = (size_t)min(tile * BM + prow, p.rows - 1) * k;
        for (int u = kCP; u * TPR < k; ++u) {
            const int t = ppart + TPR * u;
            const float v = o.cbsr_vals[base + min(t, k - 1)];
            const int c = o.cbsr_idx[base + min(t, k - 1)];
            rowp[t < k ? c : D] = rin ? v : 0.f;
        }
    };

    // A operands are read from LDS one group of four k-steps ahead of the MFMAs that consume them
    // (explicit software pipeline; the scheduling barriers keep the reads from sinking next to their use).
    auto multiply = [&](const float* b, auto sg_tag) {
        constexpr int SG = decltype(sg_tag)::value;
        if (!mm) return;
        const float* a0 = b + ((rg * SPW) * 32 + (lane & 31)) * LDA + 4 * (lane >> 5);
        float4 a[2][SPW];
#pragma unroll
        for (int j = 0; j < SPW; ++j) a[0][j] = *reinterpret_cast<const float4*>(a0 + j * 32 * LDA);
#pragma unroll
        for (int g = 0; g < KS / 4; ++g) {
            if (g + 1 < KS / 4) {
#pragma unroll
                for (int j = 0; j < SPW; ++j)
                    a[(g + 1) & 1][j] = *reinterpret_cast<const float4*>(a0 + j * 32 * LDA + 8 * (g + 1));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < SPW; ++j) {
                const float4 av = a[g & 1][j];
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av.x, breg[SG][4 * g + 0], acc[j], 0, 0, 0);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av.y, breg[SG][4 * g + 1], acc[j], 0, 0, 0);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av.z, breg[SG][4 * g + 2], acc[j], 0, 0, 0);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av.w, breg[SG][4 * g + 3], acc[j], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto clear_acc = [&]() {
#pragma unroll
        for (int j = 0; j < SPW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
    };
    auto store_tile = [&](int tile) {                  // out[rows, D] = C
        if (!mm) return;
        if (p.relu) {
#pragma unroll
            for (int j = 0; j < SPW; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[j][r] = fmaxf(acc[j][r], 0.0f);
        }
        // one pointer per sub-tile; the 16 rows a lane holds sit at fixed offsets from it
        const int row0 = tile * BM + rg * SPW * 32 + 4 * (lane >> 5);
        float* const o = p.out + (size_t)row0 * D + 32 * ct + (lane & 31);
        if (tile * BM + BM <= p.rows) {                // whole tile in range (all but the last tile)
#pragma unroll
            for (int j = 0; j < SPW; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) __builtin_nontemporal_store(acc[j][r], o + (j * 32 + 8 * (r >> 2) + (r & 3)) * D);
        } else {
#pragma unroll
            for (int j = 0; j < SPW; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = j * 32 + 8 * (r >> 2) + (r & 3);
                    if (row0 + dr < p.rows) o[dr * D] = acc[j][r];
                }
        }
    };

    if constexpr (AK == kACbsrDense) {
        // Two segments per row tile: the CBSR operand is multiplied out of buf0, the dense one out of buf1.
        const GemmOperand& oc = p.seg[0];
        PairRegs pr;
        int tile = blockIdx.x;
        load_pairs(pr, oc.cbsr_vals, oc.cbsr_idx, oc.k, tile);
        stage_cbsr(pr, tile, buf0);
        __syncthreads();
        for (;;) {
            const int ntile = tile + gridDim.x;
            const bool has_next = ntile < n_tiles;
            prefetch(tile);
            __builtin_amdgcn_sched_barrier(0);
            multiply(buf0, std::integral_constant<int, 0>{});
            __builtin_amdgcn_sched_barrier(0);
            commit(tile, buf1);
            __syncthreads();
            if (has_next) load_pairs(pr, oc.cbsr_vals, oc.cbsr_idx, oc.k, ntile);
            __builtin_amdgcn_sched_barrier(0);
            multiply(buf1, std::integral_constant<int, NSEG - 1>{});
            store_tile(tile);
            clear_acc();
            __builtin_amdgcn_sched_barrier(0);
            if (has_next) stage_cbsr(pr, ntile, buf0);
            __syncthreads();
            if (!has_next) break;
            tile = ntile;
        }
    } else {
        int tile = blockIdx.x, cur = 0;
        prefetch(tile);
        commit(tile, buf0);
        __syncthreads();
        for (;;) {
            const int ntile = tile + gridDim.x;
            const bool has_next = ntile < n_tiles;
            float* const bcur = cur ? buf1 : buf0;
            float* const bother = cur ? buf0 : buf1;
            // what the epilogue of this tile consumes is requested first, then the next tile
            PairRegs pr;
            float prev[SPW][16];
            if constexpr (EPI == kEpiSampleDense) load_pairs(pr, p.first.compact, p.first.idx, p.first.k, tile);
            if constexpr (kSample2) {
                if (p.first.compact) load_pairs(pr, p.first.compact, p.first.idx, p.first.k, tile);
                else load_cols(pr, p.first.idx, p.first.k, tile);
            }
            // C rows of this lane: row0 + j*32 + 8*(r/4) + r%4, all at fixed offsets from one pointer
            const int row0 = tile * BM + rg * SPW * 32 + 4 * (lane >> 5);
            const size_t off0 = (size_t)row0 * D + 32 * ct + (lane & 31);
            const bool full = tile * BM + BM <= p.rows;     // whole tile in range (all but the last tile)
            if constexpr (EPI == kEpiMaxMerge) {            // the other branch's values (all wavefronts)
                const float* po = p.out + off0;
                if (full) {
#pragma unroll
                    for (int j = 0; j < SPW; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) prev[j][r] = po[(j * 32 + 8 * (r >> 2) + (r & 3)) * D];
                } else {
#pragma unroll
                    for (int j = 0; j < SPW; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int row = min(row0 + j * 32 + 8 * (r >> 2) + (r & 3), p.rows - 1);
                            prev[j][r] = p.out[(size_t)row * D + 32 * ct + (lane & 31)];
                        }
                }
            }
            if (has_next) prefetch(ntile);
            __builtin_amdgcn_sched_barrier(0);   // consumers of the registers loaded above stay below the multiply
            multiply(bcur, std::integral_constant<int, 0>{});

            if constexpr (EPI == kEpiStore) {
                store_tile(tile);
            } else if constexpr (EPI == kEpiMaxMerge) {
                // mask = [near >= pinned]; out keeps the near value unless the pinned one is larger
                if (mm) {
                    float* const o = p.out + off0;
                    uint8_t* const mo = p.mask_out + off0;
#pragma unroll
                    for (int j = 0; j < SPW; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int dr = j * 32 + 8 * (r >> 2) + (r & 3);
                            const float c = acc[j][r];
                            const bool near_wins = prev[j][r] >= c;
                            // with the activation folded in, a negative near value that stays has to be rewritten too
                            const bool rewrite = !near_wins || (p.relu && prev[j][r] < 0.0f);
                            const float v = near_wins ? prev[j][r] : c;
                            if (full || row0 + dr < p.rows) {
                                mo[dr * D] = near_wins ? 1 : 0;
                                if (rewrite) o[dr * D] = p.relu ? fmaxf(v, 0.0f) : v;
                            }
                        }
                }
            } else {
                // out[row, :] = 0 except out[row, idx[row,t]] = compact[row,t] + C[row, idx[row,t]].
                // C goes to the free LDS buffer; each wavefront then rebuilds and writes its own rows.
                if (mm) {
#pragma unroll
                    for (int j = 0; j < SPW; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            bother[((rg * SPW + j) * 32 + mfma_row(lane, r)) * LDA + 32 * ct + (lane & 31)] = acc[j][r];
                }
                __syncthreads();                                   // C tile complete; bcur no longer read
                float* orow = bcur + prow * LDA;
                const float* crow = bother + prow * LDA;
                zero_own_part(orow);
                const int k = p.first.k;
#pragma unroll
                for (int u = 0; u < kCP; ++u) {
                    const int t = ppart + TPR * u;
                    const int col = t < k ? (int)pr.c[u] : D;       // pairs past k land in the padding column
                    orow[col] = pr.v[u] + crow[col];
                }
                const size_t base = (size_t)min(tile * BM + prow, p.rows - 1) * k;
                for (int u = kCP; u * TPR < k; ++u) {
                    const int t = ppart + TPR * u;
                    float v = 0.f;
                    if (!kSample2 || p.first.compact) v = p.first.compact[base + min(t, k - 1)];
                    const int c = p.first.idx[base + min(t, k - 1)];
                    const int col = t < k ? c : D;
                    orow[col] = v + crow[col];
                }
                if constexpr (kSample2) {
                    // second selection: its compact gradient is added at its own columns (the columns of one row
                    // are distinct, and a row's threads share a wavefront, so the updates do not collide)
                    if (p.second.idx) {
                        __builtin_amdgcn_wave_barrier();
                        const int k2 = p.second.k;
                        const size_t base2 = (size_t)min(tile * BM + prow, p.rows - 1) * k2;
                        // fetched here, four pairs per thread at a time: no registers held across the multiply
                        for (int u0 = 0; u0 * TPR < k2; u0 += 4) {
                            float v[4];
                            int cc[4];
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                const int t = ppart + TPR * (u0 + u);
                                v[u] = p.second.compact[base2 + min(t, k2 - 1)];
                                const int c = p.second.idx[base2 + min(t, k2 - 1)];
                                cc[u] = t < k2 ? c : D;
                            }
#pragma unroll
                            for (int u = 0; u < 4; ++u) orow[cc[u]] += v[u];
                        }
                    }
                }
                if constexpr (kSample2) {
                    // ReLU in front of the layer: the gradient of a selected input that was not positive is zero
                    // (outside the selections the row is zero anyway); the values are fetched here, late
                    for (int pass = 0; pass < 2; ++pass) {
                        const SampleSet& ss = pass ? p.second : p.first;
                        if (!ss.gate || !ss.idx) continue;
                        __builtin_amdgcn_wave_barrier();
                        const int kg = ss.k;
                        const size_t baseg = (size_t)min(tile * BM + prow, p.rows - 1) * kg;
                        for (int u0 = 0; u0 * TPR < kg; u0 += 4) {
                            float gv[4];
                            int gc[4];
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                const int t = ppart + TPR * (u0 + u);
                                gv[u] = ss.gate[baseg + min(t, kg - 1)];
                                gc[u] = t < kg ? (int)ss.idx[baseg + min(t, kg - 1)] : D;
                            }
#pragma unroll
                            for (int u = 0; u < 4; ++u)
                                if (!(gv[u] > 0.0f)) orow[gc[u]] = 0.0f;
                        }
                    }
                }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int it = 0; it < F4; ++it) {
                    const int q = it * kWave + lane;
                    const int row = wave * RPW + q / (D / 4), c4 = (q % (D / 4)) * 4;
                    const int grow = tile * BM + row;
                    const float4 v = *reinterpret_cast<const float4*>(bcur + row * LDA + c4);
                    if (grow < p.rows) { float* oo = p.out + (size_t)grow * D + c4; __builtin_nontemporal_store(v.x, oo); __builtin_nontemporal_store(v.y, oo + 1); __builtin_nontemporal_store(v.z, oo + 2); __builtin_nontemporal_store(v.w, oo + 3); }
                }
                __builtin_amdgcn_wave_barrier();
            }
            clear_acc();
            __builtin_amdgcn_sched_barrier(0);
            if (has_next) commit(ntile, bother);    // a wavefront overwrites only the C rows it has just consumed
            __syncthreads();
            if (!has_next) break;
            tile = ntile; cur ^= 1;
        }
    }
}

template <int NT, int AK, int EPI>
static int launch_proj(const GemmParams& p, hipStream_t s) {
    using C = ProjCfg<NT>;
    static std::atomic<int> resident_cache{0};         // persistent workgroups = what fits the chip at once
    int resident = resident_cache.load(std::memory_order_acquire);
    if (!resident) {                                   // concurrent first calls repeat the query: same answer
        DRC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&proj_kernel<NT, AK, EPI>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::kLds));
        int per_cu = 0, dev = 0;
        hipDeviceProp_t prop;
        DRC_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, proj_kernel<NT, AK, EPI>, kPT, C::kLds));
        DRC_HIP(hipGetDevice(&dev));
        DRC_HIP(hipGetDeviceProperties(&prop, dev));
        resident = (per_cu < 1 ? 1 : per_cu) * prop.multiProcessorCount;
        resident_cache.store(resident, std::memory_order_release);
    }
    const int n_tiles = (p.rows + C::BM - 1) / C::BM;
    int grid = resident;
    if (grid > n_tiles) grid = n_tiles;
    hipLaunchKernelGGL((proj_kernel<NT, AK, EPI>), dim3((unsigned)grid), dim3(kPT), C::kLds, s, p);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

template <int NT>
static int launch_proj_nt(const GemmParams& p, int ak, hipStream_t s) {
    const int key = ak * 10 + p.epi;
    switch (key) {
        case kADense * 10 + kEpiStore: return launch_proj<NT, kADense, kEpiStore>(p, s);
        case kADense * 10 + kEpiMaxMerge: return launch_proj<NT, kADense, kEpiMaxMerge>(p, s);
        case kADense * 10 + kEpiSampleDense: return launch_proj<NT, kADense, kEpiSampleDense>(p, s);
        case kADenseMasked * 10 + kEpiStore: return launch_proj<NT, kADenseMasked, kEpiStore>(p, s);
        case kADenseMasked * 10 + kEpiSampleDense: return launch_proj<NT, kADenseMasked, kEpiSampleDense>(p, s);
        case kADense * 10 + kEpiSampleDense2: return launch_proj<NT, kADense, kEpiSampleDense2>(p, s);
        case kADenseMasked * 10 + kEpiSampleDense2: return launch_proj<NT, kADenseMasked, kEpiSampleDense2>(p, s);
        case kACbsrDense * 10 + kEpiStore: return launch_proj<NT, kACbsrDense, kEpiStore>(p, s);
        default: return fail(DR_ERR_UNSUPPORTED, "projection operand kind %d with epilogue %d is not built", ak, p.epi);
    }
}

int launch_gemm(const GemmOperand* segs, int nseg, int64_t rows, int D, GemmEpilogue epi, float* out,
                uint8_t* mask_out, SampleSet first, SampleSet second, hipStream_t s, int relu_out) {
    if (rows == 0) return DR_OK;
    GemmParams p{};
    for (int i = 0; i < nseg; ++i) p.seg[i] = segs[i];
    p.nseg = nseg;
    p.rows = (int)rows;
    p.epi = (int)epi;
    p.out = out;
    p.mask_out = mask_out;
    p.first = first;
    p.second = second;
    p.relu = relu_out;
    if (epi == kEpiSampleDense) {
        if (first.k < 1 || !first.idx) return fail(DR_ERR_INVALID_ARG, "sampling epilogue without indices");
        if (second.idx && (second.k < 1 || !second.compact))
            return fail(DR_ERR_INVALID_ARG, "sampling epilogue: second selection without its compact gradient");
        if (second.idx || !first.compact || first.gate || second.gate) p.epi = kEpiSampleDense2;
    }
    int ak;
    if (nseg == 2) {
        if (!segs[0].cbsr_vals || !segs[0].cbsr_idx || segs[0].k < 1 || !segs[1].dense || segs[1].mask)
            return fail(DR_ERR_UNSUPPORTED, "two-segment projection expects (CBSR, unmasked dense) operands");
        ak = kACbsrDense;
    } else if (nseg == 1 && segs[0].dense) {
        ak = segs[0].mask ? kADenseMasked : kADense;
    } else {
        return fail(DR_ERR_UNSUPPORTED, "projection with %d segments / a lone CBSR operand is not built", nseg);
    }
    switch (D / 32) {
        case 1: return launch_proj_nt<1>(p, ak, s);
        case 2: return launch_proj_nt<2>(p, ak, s);
        case 3: return launch_proj_nt<3>(p, ak, s);
        case 4: return launch_proj_nt<4>(p, ak, s);
        default: return fail(DR_ERR_UNSUPPORTED, "projection width D = %d not in {32,64,96,128}", D);
    }
}

// ---------------------------------------------------------------------------------------------------
// weight gradients  dW[D,D] = A^T B  (reduction over the graph's rows).  Persistent workgroups reduce a
// contiguous slab of rows each: 16- or 32-row chunks of A and B are double-buffered through LDS (loads of the
// next chunk in flight during the multiply of the current one), the full D x D accumulator lives in MFMA
// registers (wavefront w owns row-tile w of dW), and the per-workgroup partials are summed by a second
// kernel in a fixed order (deterministic, no atomics).
// ---------------------------------------------------------------------------------------------------
// rows staged per step: 16 at D = 128 (smaller staging registers: three wavefronts per SIMD), 32 below
__host__ __device__ constexpr int wg_rows(int nt) { return nt == 4 ? 16 : 32; }
constexpr int kWgRC = 32;                  // row slabs of the workgroups are multiples of this
constexpr int kWgCP = 4;                   // CBSR pairs per thread prefetched into registers

struct WgradParams {
    WgradOperand op;
    int rows;
    int rows_per_block;
    float* scratch;
};

// AK: 0 = A dense, 1 = A as CBSR, 2 = both at once against the same B (two products, two partials: the dense
// operand's first, the CBSR operand's nb partials after it)
template <int NT, int AK, bool MASKED>
__global__ __launch_bounds__(kPT, (NT == 4 && AK != 2 ? 3 : 2)) void wgrad_partial_kernel(WgradParams p) {
    constexpr bool ADENSE = AK != 1, ACBSR = AK != 0;
    constexpr int NA = AK == 2 ? 2 : 1;          // products accumulated
    constexpr int kWgRC = wg_rows(NT);           // shadows the slab granule: rows per staged chunk here
    constexpr int kWgTPR = kPT / kWgRC;          // threads sharing one chunk row when A arrives as CBSR
    constexpr int D = NT * 32;
    constexpr int LD = D + 4;
    constexpr int F4 = kWgRC * D / 4 / kPT;      // float4 per thread per operand chunk
    constexpr int kBuf = (NA + 1) * kWgRC * LD;  // one staging buffer: dense A | B | CBSR A (when both)
    extern __shared__ __align__(16) float smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rb = blockIdx.x * p.rows_per_block;
    const int re = min(rb + p.rows_per_block, p.rows);
    const bool mm = wave < NT;                   // wavefront w owns dW rows [32w, 32w+32)
    const int prow = tid / kWgTPR, ppart = tid % kWgTPR;

    floatx16 acc[NA][NT];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][j][r] = 0.0f;

    // loads only (mask bytes raw); masking and range checks happen when the chunk is written to LDS.  Two register
    // sets: a chunk's loads are issued two chunks ahead of its multiply (a whole multiply phase lies between a load
    // and the LDS write that consumes it, which covers the memory latency under load); rows past the slab's end
    // are clamped, so every load and every LDS write is unconditional.
    struct Pre {
        float4 a[F4], b[F4];
        uint32_t m[F4];
        float pv[kWgCP];
        uint32_t pc[kWgCP];
    };
    Pre P0, P1;
    auto prefetch = [&](int rr, Pre& P) {
#pragma unroll
        for (int it = 0; it < F4; ++it) {
            const int q = it * kPT + tid;
            const int row = q / (D / 4), c4 = (q % (D / 4)) * 4;
            const size_t off = (size_t)min(rr + row, re - 1) * D + c4;
            P.b[it] = *reinterpret_cast<const float4*>(p.op.b + off);
            if (MASKED) P.m[it] = *reinterpret_cast<const uint32_t*>(p.op.b_mask + off);
            if (ADENSE) P.a[it] = *reinterpret_cast<const float4*>(p.op.a_dense + off);
        }
        if (ACBSR) {
            const int k = p.op.k;
            const size_t base = (size_t)min(rr + prow, re - 1) * k;
#pragma unroll
            for (int u = 0; u < kWgCP; ++u) {
                const int t = min(ppart + kWgTPR * u, k - 1);
                P.pv[u] = p.op.a_cbsr_vals[base + t];
                P.pc[u] = p.op.a_cbsr_idx[base + t];
            }
        }
    };
    auto commit = [&](int rr, float* buf, const Pre& P) {
        float* const sA = buf;
        float* const sB = buf + kWgRC * LD;
        float* const sC = buf + (NA == 2 ? 2 * kWgRC * LD : 0);
        const uint32_t keep = (uint32_t)p.op.b_mask_keep;
        const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int it = 0; it < F4; ++it) {
            const int q = it * kPT + tid;
            const int row = q / (D / 4), c4 = (q % (D / 4)) * 4;
            const bool in = rr + row < re;
            float4 vb = P.b[it];
            if (MASKED) {
                const uint32_t m = P.m[it];
                vb.x = (((m >> 0) & 0xffu) == keep) ? vb.x : 0.f;
                vb.y = (((m >> 8) & 0xffu) == keep) ? vb.y : 0.f;
                vb.z = (((m >> 16) & 0xffu) == keep) ? vb.z : 0.f;
                vb.w = (((m >> 24) & 0xffu) == keep) ? vb.w : 0.f;
            }
            if (!in) vb = make_float4(0.f, 0.f, 0.f, 0.f);
            *reinterpret_cast<float4*>(sB + row * LD + c4) = vb;
            if (ADENSE) {
                float4 va = P.a[it];
                if (!in) va = make_float4(0.f, 0.f, 0.f, 0.f);
                *reinterpret_cast<float4*>(sA + row * LD + c4) = va;
            }
        }
        if (ACBSR) {
            // row-owned: the kWgTPR threads of a row share a wavefront, which zeroes the row and then
            // scatters the pairs into it (LDS keeps a wavefront's accesses in order); every write is
            // unconditional, pairs past k go to the padding column
            float* rowp = sC + prow * LD;
#pragma unroll
            for (int i = 0; i < D / kWgTPR / 4; ++i)
                *reinterpret_cast<float4*>(rowp + ppart * (D / kWgTPR) + 4 * i) = z;
            __builtin_amdgcn_wave_barrier();
            const int k = p.op.k;
            const bool rin = rr + prow < re;
#pragma unroll
            for (int u = 0; u < kWgCP; ++u) {
                const int t = ppart + kWgTPR * u;
                rowp[t < k ? (int)P.pc[u] : D] = rin ? P.pv[u] : 0.f;
            }
            const size_t base = (size_t)min(rr + prow, re - 1) * k;
            for (int u = kWgCP; u * kWgTPR < k; ++u) {
                const int t = ppart + kWgTPR * u;
                const float v = p.op.a_cbsr_vals[base + min(t, k - 1)];
                const int c = p.op.a_cbsr_idx[base + min(t, k - 1)];
                rowp[t < k ? c : D] = rin ? v : 0.f;
            }
        }
    };
    auto multiply = [&](const float* buf) {
        if (mm) {
            // operands of k-step i+1 are read from LDS before the MFMAs of k-step i are issued
            const float* pa = buf + (lane >> 5) * LD + wave * 32 + (lane & 31);
            const float* pb = buf + kWgRC * LD + (lane >> 5) * LD + (lane & 31);
            float av[2][NA], b[2][NT];
#pragma unroll
            for (int a = 0; a < NA; ++a) av[0][a] = pa[a * 2 * kWgRC * LD];
#pragma unroll
            for (int j = 0; j < NT; ++j) b[0][j] = pb[j * 32];
#pragma unroll
            for (int i = 0; i < kWgRC / 2; ++i) {
                if (i + 1 < kWgRC / 2) {
#pragma unroll
                    for (int a = 0; a < NA; ++a) av[(i + 1) & 1][a] = pa[a * 2 * kWgRC * LD + (2 * i + 2) * LD];
#pragma unroll
                    for (int j = 0; j < NT; ++j) b[(i + 1) & 1][j] = pb[(2 * i + 2) * LD + j * 32];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int a = 0; a < NA; ++a)
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[a][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i & 1][a], b[i & 1][j], acc[a][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    if (rb < re) {
        float* const buf0 = smem;
        float* const buf1 = smem + kBuf;
        prefetch(rb, P0);
        prefetch(rb + kWgRC, P1);
        commit(rb, buf0, P0);
        __syncthreads();
        // buf0 holds chunk rr, P1 the loads of chunk rr + kWgRC; sched_barriers keep the consumers of the
        // prefetched registers below the multiply
        // (two chunks per trip, one exit at the bottom: the register sets stay where they are across the back edge;
        // a slab with an odd number of chunks stages one chunk of zeros and skips its multiply)
        int rr = rb;
        do {
            prefetch(rr + 2 * kWgRC, P0);
            __builtin_amdgcn_sched_barrier(0);
            multiply(buf0);
            __builtin_amdgcn_sched_barrier(0);
            commit(rr + kWgRC, buf1, P1);
            __syncthreads();
            prefetch(rr + 3 * kWgRC, P1);
            __builtin_amdgcn_sched_barrier(0);
            if (rr + kWgRC < re) multiply(buf1);
            __builtin_amdgcn_sched_barrier(0);
            commit(rr + 2 * kWgRC, buf0, P0);
            __syncthreads();
            rr += 2 * kWgRC;
        } while (rr < re);
    }

    if (mm) {
#pragma unroll
        for (int a = 0; a < NA; ++a) {
            float* out = p.scratch + ((size_t)a * gridDim.x + blockIdx.x) * D * D;
#pragma unroll
            for (int j = 0; j < NT; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    out[(size_t)(wave * 32 + mfma_row(lane, r)) * D + j * 32 + (lane & 31)] = acc[a][j][r];
        }
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
    if (q < dd) {
        // eight loads in flight at a time (the adds keep their order): the kernel is bound by load latency otherwise
        int b = wave;
        for (; b + 56 < nb; b += 64) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = scratch[(size_t)(b + 8 * u) * dd + q];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; b < nb; b += 8) s += scratch[(size_t)b * dd + q];
    }
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

// room for the two partial sets of a paired launch
size_t wgrad_scratch_bytes(int64_t rows, int D) { return sizeof(float) * 2 * (size_t)wgrad_blocks(rows) * D * D; }

template <int NT, int AK, bool MASKED>
static int launch_wgrad_kernel(const WgradParams& p, int nb, hipStream_t s) {
    constexpr size_t lds = sizeof(float) * 2 * (AK == 2 ? 3 : 2) * wg_rows(NT) * (NT * 32 + 4);
    static std::atomic<bool> configured{false};
    if (!configured.load(std::memory_order_acquire)) {
        DRC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_partial_kernel<NT, AK, MASKED>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        configured.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((wgrad_partial_kernel<NT, AK, MASKED>), dim3((unsigned)nb), dim3(kPT), lds, s, p);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

template <int NT>
static int launch_wgrad_nt(const WgradParams& p, int nb, hipStream_t s) {
    const bool dense = p.op.a_dense != nullptr, cbsr = p.op.a_cbsr_vals != nullptr, masked = p.op.b_mask != nullptr;
    if (dense && cbsr) return masked ? launch_wgrad_kernel<NT, 2, true>(p, nb, s) : launch_wgrad_kernel<NT, 2, false>(p, nb, s);
    if (cbsr) return masked ? launch_wgrad_kernel<NT, 1, true>(p, nb, s) : launch_wgrad_kernel<NT, 1, false>(p, nb, s);
    return masked ? launch_wgrad_kernel<NT, 0, true>(p, nb, s) : launch_wgrad_kernel<NT, 0, false>(p, nb, s);
}

// dW = A^T B.  With both a dense and a CBSR A operand in `op` the two products are formed in one pass over B:
// the dense operand's goes to dW, the CBSR operand's to dW_cbsr (unused otherwise).
int launch_wgrad(const WgradOperand& op, int64_t rows, int D, float* dW, float* dW_cbsr, void* scratch, hipStream_t s) {
    const bool cbsr = op.a_cbsr_vals != nullptr;
    if (cbsr && (!op.a_cbsr_idx || op.k < 1)) return fail(DR_ERR_INVALID_ARG, "weight gradient: incomplete CBSR operand");
    if (!op.a_dense && !cbsr) return fail(DR_ERR_INVALID_ARG, "weight gradient without an A operand");
    const bool pair = op.a_dense && cbsr;
    if (pair && !dW_cbsr) return fail(DR_ERR_INVALID_ARG, "paired weight gradient without its second output");
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
    if (pair)
        hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((dd + 63) / 64)), dim3(512), 0, s,
                           static_cast<float*>(scratch) + (size_t)nb * dd, nb, dd, dW_cbsr);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

}  // namespace drc
