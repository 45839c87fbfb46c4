// DR-SpMM forward (paper Section 3.2 / Alg. 1) and backward (Section 3.3 / Alg. 2) for one relation.
//
// Work decomposition (both directions).  A workgroup owns a block of kRowsPerBlock consecutive CSR rows.
//   * The wavefront is split into groups of 8 lanes; a group owns one row at a time and walks that row's
//     edges in storage order, so 8 rows are in flight per wavefront (the wave64 counterpart of the paper's
//     "partition the warp into parts, one neighbour each") and a row's sum has one fixed order: results
//     are reproducible bit for bit.
//   * Rows of the block are counting-sorted by degree in LDS first (integer LDS atomics), and the 8 rows
//     a wavefront takes together are neighbours in that order: the groups of a wavefront run the same
//     number of edge iterations (the paper's degree classes, resolved per block).
//   * Rows with more than kLongRow edges (high-fanout nets) are not given to one group: the whole
//     workgroup strides over their edges into per-group partial sums that are then added in a fixed order.
//   * Workgroup ids are remapped so each XCD walks a contiguous range of row blocks: neighbouring rows of
//     the spatially local `near` relation gather overlapping source rows, which then hit in that XCD's L2.
//
// Forward.  Lane t of a group loads pairs [t*k/8, (t+1)*k/8) of the gathered source row with vector
// loads (one 128-byte line of values per source row at k = 32) and adds a*v into the group's private
// LDS row buffer with plain read-modify-write: the pairs of one source row have distinct columns and
// no other group touches the buffer, so no atomics are needed (ds_add_f32 is far slower than plain LDS
// traffic on this chip).  The finished row goes to HBM in 128-byte segments.
//
// Backward.  Lane t of a group owns the compact outputs t, t+8, t+16, ... of its source row and keeps
// them in registers; per edge it reads dH[destination, idx[slot]] directly (the interleaved slot
// assignment keeps the 8 lanes of one load inside one 128-byte line of the dH row when k*4 = D).
#include "dr_internal.h"

namespace drc {

constexpr int kLPE = 8;             // lanes per row group
constexpr int kLongRow = 256;       // rows with more edges are processed by the whole workgroup
constexpr int kRowsPerBlock = 256;
constexpr int kBins = kLongRow + 1;

struct BlockPlan {
    int* sRp;      // [kRowsPerBlock + 1] row pointers of the block
    int* sOrder;   // [kRowsPerBlock] short rows, degree descending
    int* sHist;    // [kBins + 1]
    int* sLong;    // [kRowsPerBlock] long rows
    int* sCnt;     // [4]: number of long rows
};

__host__ __device__ constexpr int plan_ints() { return (kRowsPerBlock + 1) + kRowsPerBlock + (kBins + 1) + kRowsPerBlock + 4; }

__device__ __forceinline__ BlockPlan carve_plan(int* base) {
    BlockPlan p;
    p.sRp = base;
    p.sOrder = p.sRp + (kRowsPerBlock + 1);
    p.sHist = p.sOrder + kRowsPerBlock;
    p.sLong = p.sHist + (kBins + 1);
    p.sCnt = p.sLong + kRowsPerBlock;
    return p;
}

// Loads the block's row pointers and sorts its rows by degree (descending).  Returns the number of
// short rows; p.sCnt[0] holds the number of long rows.  Ends with a barrier.
__device__ __forceinline__ int plan_block(const BlockPlan& p, const int32_t* __restrict__ rowptr, int r0, int nr) {
    const int tid = threadIdx.x, bd = blockDim.x;
    for (int i = tid; i <= nr; i += bd) p.sRp[i] = rowptr[r0 + i];
    for (int i = tid; i <= kBins; i += bd) p.sHist[i] = 0;
    if (tid < 4) p.sCnt[tid] = 0;
    __syncthreads();
    for (int i = tid; i < nr; i += bd) {
        int deg = p.sRp[i + 1] - p.sRp[i];
        if (deg > kLongRow) p.sLong[atomicAdd(&p.sCnt[0], 1)] = i;
        else atomicAdd(&p.sHist[kLongRow - deg], 1);        // bin 0 = largest degree
    }
    __syncthreads();
    if (tid < kWave) {                                       // exclusive scan of the bins by one wavefront
        constexpr int kPer = (kBins + kWave - 1) / kWave;
        int c[kPer], s = 0;
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
            int b = tid * kPer + q;
            c[q] = (b < kBins) ? p.sHist[b] : 0;
            s += c[q];
        }
        int incl = s;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            int y = __shfl_up(incl, d, kWave);
            if (tid >= d) incl += y;
        }
        int excl = incl - s;
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
            int b = tid * kPer + q;
            if (b < kBins) p.sHist[b] = excl;
            excl += c[q];
        }
    }
    __syncthreads();
    for (int i = tid; i < nr; i += bd) {
        int deg = p.sRp[i + 1] - p.sRp[i];
        if (deg <= kLongRow) p.sOrder[atomicAdd(&p.sHist[kLongRow - deg], 1)] = i;
    }
    __syncthreads();
    return nr - p.sCnt[0];
}

// ---------------------------------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------------------------------

template <int KPL> struct Pairs {        // KPL consecutive (value, column) pairs of one CBSR row
    float v[KPL];
    uint16_t c[KPL];
    __device__ __forceinline__ void load(const float* __restrict__ vals, const uint16_t* __restrict__ idx, uint32_t off) {
        if constexpr (KPL == 1) {
            v[0] = vals[off];
            c[0] = idx[off];
        } else if constexpr (KPL == 2) {
            float2 a = *reinterpret_cast<const float2*>(vals + off);
            ushort2 b = *reinterpret_cast<const ushort2*>(idx + off);
            v[0] = a.x; v[1] = a.y; c[0] = b.x; c[1] = b.y;
        } else {
#pragma unroll
            for (int q = 0; q < KPL / 4; ++q) {
                float4 a = *reinterpret_cast<const float4*>(vals + off + 4 * q);
                ushort4 b = *reinterpret_cast<const ushort4*>(idx + off + 4 * q);
                v[4 * q + 0] = a.x; v[4 * q + 1] = a.y; v[4 * q + 2] = a.z; v[4 * q + 3] = a.w;
                c[4 * q + 0] = b.x; c[4 * q + 1] = b.y; c[4 * q + 2] = b.z; c[4 * q + 3] = b.w;
            }
        }
    }
    // buf[c] += a * v for all pairs; the columns of one CBSR row are distinct, so the reads can all be
    // issued before the writes
    __device__ __forceinline__ void accumulate(float* buf, float a) const {
        float old[KPL];
#pragma unroll
        for (int u = 0; u < KPL; ++u) old[u] = buf[c[u]];
#pragma unroll
        for (int u = 0; u < KPL; ++u) buf[c[u]] = fmaf(a, v[u], old[u]);
    }
};

// One group walks edges e, e+stride, ... < e_end of its row, software-pipelined three deep: edge record
// (column, value) -> gather of the source row's pairs -> LDS accumulation.  All 64 lanes stay in the
// loop until every group of the wavefront is done.
template <int KPL>
__device__ __forceinline__ void fwd_walk(const int32_t* __restrict__ colidx, const float* __restrict__ avals,
                                         const float* __restrict__ xs_vals, const uint16_t* __restrict__ xs_idx,
                                         int e, int e_end, int stride, int k, int t, float* buf) {
    if constexpr (KPL > 0) {
        bool valid1 = e < e_end, valid2 = false;
        int col1 = 0;
        float a1 = 0.f, a2 = 0.f;
        if (valid1) { col1 = colidx[e]; a1 = avals[e]; }
        e += stride;
        Pairs<KPL> p2;
        while (__any(valid1 || valid2)) {
            Pairs<KPL> pn;
            const bool validn = valid1;
            const float an = a1;
            if (valid1) pn.load(xs_vals, xs_idx, (uint32_t)col1 * (uint32_t)k + (uint32_t)(t * KPL));
            valid1 = e < e_end;
            if (valid1) { col1 = colidx[e]; a1 = avals[e]; }
            e += stride;
            if (valid2) p2.accumulate(buf, a2);
            if (validn) p2 = pn;
            a2 = an;
            valid2 = validn;
        }
    } else {
        // generic k: lane t takes pairs t, t+8, ... with scalar loads
        for (; __any(e < e_end); e += stride) {
            if (e < e_end) {
                const uint32_t base = (uint32_t)colidx[e] * (uint32_t)k;
                const float a = avals[e];
                for (int s = t; s < k; s += kLPE) {
                    const int c = xs_idx[base + s];
                    buf[c] = fmaf(a, xs_vals[base + s], buf[c]);
                }
            }
        }
    }
}

template <int KPL>
__global__ __launch_bounds__(256) void spmm_fwd_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx, const float* __restrict__ avals,
    const float* __restrict__ xs_vals, const uint16_t* __restrict__ xs_idx, float* __restrict__ H,
    int M, int D, int k, int n_tiles, int per_xcd, int vec_store) {
    extern __shared__ float4 smem4[];
    float* rowbuf = reinterpret_cast<float*>(smem4);                 // [groups][D], 16-byte aligned
    const int groups = blockDim.x / kLPE;
    BlockPlan plan = carve_plan(reinterpret_cast<int*>(rowbuf + groups * D));

    const int tile_id = xcd_contiguous_tile(blockIdx.x, per_xcd);
    if (tile_id >= n_tiles) return;
    const int r0 = tile_id * kRowsPerBlock;
    const int nr = min(kRowsPerBlock, M - r0);
    const int tid = threadIdx.x;
    const int g = tid / kLPE, t = tid % kLPE;
    float* buf = rowbuf + g * D;

    for (int i = tid; i < groups * D; i += blockDim.x) rowbuf[i] = 0.0f;
    const int n_short = plan_block(plan, rowptr, r0, nr);   // barriers inside
    const int n_long = plan.sCnt[0];

    // ---- rows with very many edges: the whole workgroup, partial sums per group ----
    for (int li = 0; li < n_long; ++li) {
        const int row = plan.sLong[li];
        fwd_walk<KPL>(colidx, avals, xs_vals, xs_idx, plan.sRp[row] + g, plan.sRp[row + 1], groups, k, t, buf);
        __syncthreads();
        float* out = H + (size_t)(r0 + row) * D;
        for (int c = tid; c < D; c += blockDim.x) {
            float s = 0.0f;
            for (int q = 0; q < groups; ++q) {
                s += rowbuf[q * D + c];
                rowbuf[q * D + c] = 0.0f;
            }
            out[c] = s;
        }
        __syncthreads();
    }

    // ---- all other rows: one group per row, 8 rows of similar degree per wavefront ----
    for (int slot = g; slot < n_short + (kWave / kLPE - 1); slot += groups) {
        const bool has = slot < n_short;
        if (!__any(has)) break;
        const int row = has ? plan.sOrder[slot] : 0;
        const int e0 = has ? plan.sRp[row] : 0;
        const int e1 = has ? plan.sRp[row + 1] : 0;
        fwd_walk<KPL>(colidx, avals, xs_vals, xs_idx, e0, e1, 1, k, t, buf);
        if (has) {
            float* out = H + (size_t)(r0 + row) * D;
            if (vec_store) {
                for (int c = t * 4; c < D; c += kLPE * 4) {
                    float4 v = *reinterpret_cast<const float4*>(buf + c);
                    *reinterpret_cast<float4*>(out + c) = v;
                    *reinterpret_cast<float4*>(buf + c) = make_float4(0.f, 0.f, 0.f, 0.f);
                }
            } else {
                for (int c = t; c < D; c += kLPE) {
                    out[c] = buf[c];
                    buf[c] = 0.0f;
                }
            }
        }
    }
}

static int spmm_block_threads(int D) { return D <= 256 ? 256 : (D <= 512 ? 128 : 64); }

int launch_spmm_fwd(const dr_csr* A, const float* xs_vals, const uint16_t* xs_idx, int D, int k, float* H,
                    hipStream_t s) {
    const int M = (int)A->n_rows;
    const int n_tiles = (M + kRowsPerBlock - 1) / kRowsPerBlock;
    const int per_xcd = (n_tiles + kNumXcd - 1) / kNumXcd;
    const int threads = spmm_block_threads(D);
    const int groups = threads / kLPE;
    const int vec_store = (D % 4 == 0 && aligned(H, 16)) ? 1 : 0;
    int kpl = 0;
    if (k % kLPE == 0) {
        const int q = k / kLPE;
        if (q == 1) kpl = 1;
        else if (q == 2 && aligned(xs_vals, 8) && aligned(xs_idx, 4)) kpl = 2;
        else if ((q == 4 || q == 8 || q == 16) && aligned(xs_vals, 16) && aligned(xs_idx, 8)) kpl = q;
    }
    const size_t lds = sizeof(float) * (size_t)groups * D + sizeof(int) * (size_t)plan_ints();
    dim3 grid((unsigned)(per_xcd * kNumXcd)), block((unsigned)threads);
#define DRC_LAUNCH_FWD(V)                                                                                      \
    hipLaunchKernelGGL(spmm_fwd_kernel<V>, grid, block, lds, s, A->rowptr, A->colidx, A->vals, xs_vals, xs_idx, \
                       H, M, D, k, n_tiles, per_xcd, vec_store)
    switch (kpl) {
        case 1: DRC_LAUNCH_FWD(1); break;
        case 2: DRC_LAUNCH_FWD(2); break;
        case 4: DRC_LAUNCH_FWD(4); break;
        case 8: DRC_LAUNCH_FWD(8); break;
        case 16: DRC_LAUNCH_FWD(16); break;
        default: DRC_LAUNCH_FWD(0); break;
    }
#undef DRC_LAUNCH_FWD
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

// ---------------------------------------------------------------------------------------------------
// backward: rows are sources j (rows of A^T); lane t of the row's group owns compact slots
// s0 + t, s0 + t + 8, ... (KPL of them) in registers.  k larger than 8*KPL is covered by re-walking the
// row for the next window of slots.
// ---------------------------------------------------------------------------------------------------

template <int KPL>
__device__ __forceinline__ void bwd_walk(const int32_t* __restrict__ colidx, const float* __restrict__ avals,
                                         const float* __restrict__ dH, int D, int e, int e_end, int stride,
                                         const int (&ci)[KPL], float (&acc)[KPL]) {
    bool valid1 = e < e_end, valid2 = false;
    int col1 = 0;
    float a1 = 0.f, a2 = 0.f;
    if (valid1) { col1 = colidx[e]; a1 = avals[e]; }
    e += stride;
    float v2[KPL];
#pragma unroll
    for (int u = 0; u < KPL; ++u) v2[u] = 0.f;
    while (__any(valid1 || valid2)) {
        float vn[KPL];
        const bool validn = valid1;
        const float an = a1;
        if (valid1) {
            const float* rowp = dH + (size_t)(uint32_t)col1 * (uint32_t)D;
#pragma unroll
            for (int u = 0; u < KPL; ++u) vn[u] = rowp[ci[u]];
        }
        valid1 = e < e_end;
        if (valid1) { col1 = colidx[e]; a1 = avals[e]; }
        e += stride;
        if (valid2) {
#pragma unroll
            for (int u = 0; u < KPL; ++u) acc[u] = fmaf(a2, v2[u], acc[u]);
        }
        if (validn) {
#pragma unroll
            for (int u = 0; u < KPL; ++u) v2[u] = vn[u];
        }
        a2 = an;
        valid2 = validn;
    }
}

template <int KPL>
__global__ __launch_bounds__(256) void spmm_bwd_kernel(
    const int32_t* __restrict__ t_rowptr, const int32_t* __restrict__ t_colidx, const float* __restrict__ t_vals,
    const float* __restrict__ dH, const uint16_t* __restrict__ xs_idx, float* __restrict__ dXs,
    int N, int D, int k, int n_tiles, int per_xcd, int accumulate) {
    extern __shared__ float4 smem4[];
    constexpr int kWin = kLPE * KPL;                                   // compact slots per pass
    constexpr int kGroups = 256 / kLPE;
    float* part = reinterpret_cast<float*>(smem4);                     // [kGroups][kWin] long-row partials
    BlockPlan plan = carve_plan(reinterpret_cast<int*>(part + kGroups * kWin));

    const int tile_id = xcd_contiguous_tile(blockIdx.x, per_xcd);
    if (tile_id >= n_tiles) return;
    const int r0 = tile_id * kRowsPerBlock;
    const int nr = min(kRowsPerBlock, N - r0);
    const int tid = threadIdx.x;
    const int g = tid / kLPE, t = tid % kLPE;

    const int n_short = plan_block(plan, t_rowptr, r0, nr);
    const int n_long = plan.sCnt[0];

    for (int s0 = 0; s0 < k; s0 += kWin) {
        // ---- long rows ----
        for (int li = 0; li < n_long; ++li) {
            const int row = plan.sLong[li];
            const uint16_t* ridx = xs_idx + (size_t)(r0 + row) * k;
            int ci[KPL];
            float acc[KPL];
#pragma unroll
            for (int u = 0; u < KPL; ++u) {
                const int slot = s0 + t + kLPE * u;
                ci[u] = (slot < k) ? ridx[slot] : 0;
                acc[u] = 0.f;
            }
            bwd_walk<KPL>(t_colidx, t_vals, dH, D, plan.sRp[row] + g, plan.sRp[row + 1], kGroups, ci, acc);
#pragma unroll
            for (int u = 0; u < KPL; ++u) part[g * kWin + t + kLPE * u] = acc[u];
            __syncthreads();
            for (int w = tid; w < kWin; w += 256) {
                const int slot = s0 + w;
                if (slot < k) {
                    float s = 0.f;
                    for (int q = 0; q < kGroups; ++q) s += part[q * kWin + w];
                    float* o = dXs + (size_t)(r0 + row) * k + slot;
                    *o = accumulate ? (*o + s) : s;
                }
            }
            __syncthreads();
        }
        // ---- short rows ----
        for (int slot_r = g; slot_r < n_short + (kWave / kLPE - 1); slot_r += kGroups) {
            const bool has = slot_r < n_short;
            if (!__any(has)) break;
            const int row = has ? plan.sOrder[slot_r] : 0;
            const int e0 = has ? plan.sRp[row] : 0;
            const int e1 = has ? plan.sRp[row + 1] : 0;
            const uint16_t* ridx = xs_idx + (size_t)(r0 + row) * k;
            int ci[KPL];
            float acc[KPL];
#pragma unroll
            for (int u = 0; u < KPL; ++u) {
                const int slot = s0 + t + kLPE * u;
                ci[u] = (has && slot < k) ? ridx[slot] : 0;
                acc[u] = 0.f;
            }
            bwd_walk<KPL>(t_colidx, t_vals, dH, D, e0, e1, 1, ci, acc);
            if (has) {
                float* o = dXs + (size_t)(r0 + row) * k;
#pragma unroll
                for (int u = 0; u < KPL; ++u) {
                    const int slot = s0 + t + kLPE * u;
                    if (slot < k) o[slot] = accumulate ? (o[slot] + acc[u]) : acc[u];
                }
            }
        }
    }
}

int launch_spmm_bwd(const dr_csr* At, const float* dH, const uint16_t* xs_idx, int D, int k, float* dXs,
                    int accumulate, hipStream_t s) {
    const int N = (int)At->n_rows;
    const int n_tiles = (N + kRowsPerBlock - 1) / kRowsPerBlock;
    const int per_xcd = (n_tiles + kNumXcd - 1) / kNumXcd;
    int kpl = 8;
    if (k <= 8) kpl = 1;
    else if (k <= 16) kpl = 2;
    else if (k <= 32) kpl = 4;
    dim3 grid((unsigned)(per_xcd * kNumXcd)), block(256);
    const size_t lds = sizeof(float) * (size_t)(256 / kLPE) * (kLPE * kpl) + sizeof(int) * (size_t)plan_ints();
#define DRC_LAUNCH_BWD(V)                                                                                       \
    hipLaunchKernelGGL(spmm_bwd_kernel<V>, grid, block, lds, s, At->rowptr, At->colidx, At->vals, dH, xs_idx, dXs, \
                       N, D, k, n_tiles, per_xcd, accumulate ? 1 : 0)
    switch (kpl) {
        case 1: DRC_LAUNCH_BWD(1); break;
        case 2: DRC_LAUNCH_BWD(2); break;
        case 4: DRC_LAUNCH_BWD(4); break;
        default: DRC_LAUNCH_BWD(8); break;
    }
#undef DRC_LAUNCH_BWD
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

}  // namespace drc
