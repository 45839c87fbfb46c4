// DR-SpMM forward (paper Section 3.2 / Alg. 1) and backward (Section 3.3 / Alg. 2) for one relation.
//
// Both kernels give one workgroup a tile of R consecutive CSR rows and walk the tile's edges as one
// flat range, so the work per workgroup is proportional to its edge count and a high-fanout row is
// simply a longer range shared by all 256 lanes (no row is bound to a single wavefront).
//
//  * edges are staged in LDS in chunks: (source column, edge value, local row) per edge, loaded with
//    coalesced reads; the local row comes from a binary search in the tile's row pointers;
//  * a group of LPE lanes owns one staged edge at a time and gathers that source row's k surviving
//    (value, column) pairs with vector loads; 256/LPE edges are in flight per workgroup step -- the
//    wave64 counterpart of the paper's "ceil(32/K) parts per warp";
//  * contributions are accumulated into an LDS tile with ds_add_f32 (pairs of one edge never collide;
//    pairs of different edges of the same row may, which the LDS atomic unit resolves);
//  * the finished tile is one contiguous block of the output and is written with coalesced stores.
//
// Workgroup ids are remapped so that each XCD walks a contiguous range of row tiles: neighbouring rows
// of the spatially local `near` relation gather overlapping source rows, which then hit in that XCD's L2.
#include "dr_internal.h"

namespace drc {

constexpr int kThreads = 256;
constexpr int kChunk = 512;  // edges staged per pass

__device__ __forceinline__ void lds_add(float* p, float v) {
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

template <int VEC> struct PairVec;
template <> struct PairVec<1> {
    float v[1]; uint16_t c[1];
    __device__ __forceinline__ void load(const float* vals, const uint16_t* idx, uint32_t off) {
        v[0] = vals[off]; c[0] = idx[off];
    }
};
template <> struct PairVec<2> {
    float v[2]; uint16_t c[2];
    __device__ __forceinline__ void load(const float* vals, const uint16_t* idx, uint32_t off) {
        float2 a = *reinterpret_cast<const float2*>(vals + off);
        ushort2 b = *reinterpret_cast<const ushort2*>(idx + off);
        v[0] = a.x; v[1] = a.y; c[0] = b.x; c[1] = b.y;
    }
};
template <> struct PairVec<4> {
    float v[4]; uint16_t c[4];
    __device__ __forceinline__ void load(const float* vals, const uint16_t* idx, uint32_t off) {
        float4 a = *reinterpret_cast<const float4*>(vals + off);
        ushort4 b = *reinterpret_cast<const ushort4*>(idx + off);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        c[0] = b.x; c[1] = b.y; c[2] = b.z; c[3] = b.w;
    }
};

// stage edges [c0, c0+n) of the tile: column, value and local row (largest lr with sRp[lr] <= e)
__device__ __forceinline__ void stage_edges(const int32_t* __restrict__ colidx, const float* __restrict__ avals,
                                            int c0, int n, const int* sRp, int nr, int* sCol, float* sA, int* sRow) {
    for (int i = threadIdx.x; i < n; i += kThreads) {
        int e = c0 + i;
        sCol[i] = colidx[e];
        sA[i] = avals[e];
        int lo = 0, hi = nr;
        while (hi - lo > 1) {
            int mid = (lo + hi) >> 1;
            if (sRp[mid] <= e) lo = mid; else hi = mid;
        }
        sRow[i] = lo;
    }
}

template <int VEC>
__global__ __launch_bounds__(kThreads) void spmm_fwd_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx, const float* __restrict__ avals,
    const float* __restrict__ xs_vals, const uint16_t* __restrict__ xs_idx, float* __restrict__ H,
    int M, int D, int k, int R, int lpe_log2, int n_tiles, int per_xcd, int vec_store) {
    extern __shared__ float smem[];
    float* tile = smem;                                   // [R*D]
    int* sRp = reinterpret_cast<int*>(tile + R * D);      // [R+1]
    int* sCol = sRp + (R + 1);                            // [kChunk]
    float* sA = reinterpret_cast<float*>(sCol + kChunk);  // [kChunk]
    int* sRow = reinterpret_cast<int*>(sA + kChunk);      // [kChunk]

    const int tile_id = xcd_contiguous_tile(blockIdx.x, per_xcd);
    if (tile_id >= n_tiles) return;
    const int r0 = tile_id * R;
    const int nr = min(R, M - r0);
    const int tid = threadIdx.x;

    for (int i = tid; i <= nr; i += kThreads) sRp[i] = rowptr[r0 + i];
    for (int i = tid; i < nr * D; i += kThreads) tile[i] = 0.0f;
    __syncthreads();

    const int e_begin = sRp[0], e_end = sRp[nr];
    const int lpe = 1 << lpe_log2;
    const int groups = kThreads >> lpe_log2;
    const int g = tid >> lpe_log2;
    const int t0 = (tid & (lpe - 1)) * VEC;
    const int t_step = lpe * VEC;

    for (int c0 = e_begin; c0 < e_end; c0 += kChunk) {
        const int n = min(kChunk, e_end - c0);
        stage_edges(colidx, avals, c0, n, sRp, nr, sCol, sA, sRow);
        __syncthreads();
        for (int t = t0; t < k; t += t_step) {
            int i = g;
            for (; i + groups < n; i += 2 * groups) {   // two edges in flight per group
                const int i2 = i + groups;
                PairVec<VEC> p, q;
                p.load(xs_vals, xs_idx, (uint32_t)sCol[i] * (uint32_t)k + (uint32_t)t);
                q.load(xs_vals, xs_idx, (uint32_t)sCol[i2] * (uint32_t)k + (uint32_t)t);
                const float a = sA[i], b = sA[i2];
                float* rp = tile + sRow[i] * D;
                float* rq = tile + sRow[i2] * D;
#pragma unroll
                for (int u = 0; u < VEC; ++u) lds_add(rp + p.c[u], a * p.v[u]);
#pragma unroll
                for (int u = 0; u < VEC; ++u) lds_add(rq + q.c[u], b * q.v[u]);
            }
            if (i < n) {
                PairVec<VEC> p;
                p.load(xs_vals, xs_idx, (uint32_t)sCol[i] * (uint32_t)k + (uint32_t)t);
                const float a = sA[i];
                float* rp = tile + sRow[i] * D;
#pragma unroll
                for (int u = 0; u < VEC; ++u) lds_add(rp + p.c[u], a * p.v[u]);
            }
        }
        __syncthreads();
    }

    float* out = H + (size_t)r0 * D;
    const int total = nr * D;
    if (vec_store) {
        const float4* t4 = reinterpret_cast<const float4*>(tile);
        float4* o4 = reinterpret_cast<float4*>(out);
        for (int i = tid; i < (total >> 2); i += kThreads) o4[i] = t4[i];
    } else {
        for (int i = tid; i < total; i += kThreads) out[i] = tile[i];
    }
}

static int pow2_ceil_log2(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

int launch_spmm_fwd(const dr_csr* A, const float* xs_vals, const uint16_t* xs_idx, int D, int k, float* H,
                    hipStream_t s) {
    const int M = (int)A->n_rows;
    int R = 4096 / D;
    if (R < 1) R = 1;
    if (R > 64) R = 64;
    const int n_tiles = (M + R - 1) / R;
    const int per_xcd = (n_tiles + kNumXcd - 1) / kNumXcd;
    int vec = 1;
    if (k % 4 == 0 && aligned(xs_vals, 16) && aligned(xs_idx, 8)) vec = 4;
    else if (k % 2 == 0 && aligned(xs_vals, 8) && aligned(xs_idx, 4)) vec = 2;
    int lpe_log2 = pow2_ceil_log2((k + vec - 1) / vec);
    if (lpe_log2 > 8) lpe_log2 = 8;
    const int vec_store = (D % 4 == 0 && aligned(H, 16)) ? 1 : 0;
    const size_t lds = sizeof(float) * (size_t)R * D + sizeof(int) * (size_t)(R + 1 + 3 * kChunk);
    dim3 grid((unsigned)(per_xcd * kNumXcd)), block(kThreads);
#define DRC_LAUNCH_FWD(V)                                                                                      \
    hipLaunchKernelGGL(spmm_fwd_kernel<V>, grid, block, lds, s, A->rowptr, A->colidx, A->vals, xs_vals, xs_idx, \
                       H, M, D, k, R, lpe_log2, n_tiles, per_xcd, vec_store)
    if (vec == 4) DRC_LAUNCH_FWD(4);
    else if (vec == 2) DRC_LAUNCH_FWD(2);
    else DRC_LAUNCH_FWD(1);
#undef DRC_LAUNCH_FWD
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

// ---------------------------------------------------------------------------------------------------
// backward: rows are sources j (rows of A^T); the output tile is compact [R, k]; lane t of a group
// reads dH[destination, idx[j,t]] for its staged edge.
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void spmm_bwd_kernel(
    const int32_t* __restrict__ t_rowptr, const int32_t* __restrict__ t_colidx, const float* __restrict__ t_vals,
    const float* __restrict__ dH, const uint16_t* __restrict__ xs_idx, float* __restrict__ dXs,
    int N, int D, int k, int R, int lpe_log2, int n_tiles, int per_xcd, int accumulate) {
    extern __shared__ float smem[];
    float* tile = smem;                                   // [R*k]
    int* sRp = reinterpret_cast<int*>(tile + R * k);      // [R+1]
    int* sCol = sRp + (R + 1);                            // [kChunk]
    float* sA = reinterpret_cast<float*>(sCol + kChunk);  // [kChunk]
    int* sRow = reinterpret_cast<int*>(sA + kChunk);      // [kChunk]
    uint16_t* sIdx = reinterpret_cast<uint16_t*>(sRow + kChunk);  // [R*k]

    const int tile_id = xcd_contiguous_tile(blockIdx.x, per_xcd);
    if (tile_id >= n_tiles) return;
    const int r0 = tile_id * R;
    const int nr = min(R, N - r0);
    const int tid = threadIdx.x;

    for (int i = tid; i <= nr; i += kThreads) sRp[i] = t_rowptr[r0 + i];
    const uint16_t* gidx = xs_idx + (size_t)r0 * k;
    for (int i = tid; i < nr * k; i += kThreads) {
        tile[i] = 0.0f;
        sIdx[i] = gidx[i];
    }
    __syncthreads();

    const int e_begin = sRp[0], e_end = sRp[nr];
    const int lpe = 1 << lpe_log2;
    const int groups = kThreads >> lpe_log2;
    const int g = tid >> lpe_log2;
    const int t0 = tid & (lpe - 1);

    for (int c0 = e_begin; c0 < e_end; c0 += kChunk) {
        const int n = min(kChunk, e_end - c0);
        stage_edges(t_colidx, t_vals, c0, n, sRp, nr, sCol, sA, sRow);
        __syncthreads();
        for (int t = t0; t < k; t += lpe) {
            int i = g;
            for (; i + 3 * groups < n; i += 4 * groups) {   // four edges in flight per group
                float v[4], a[4];
                int slot[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int iu = i + u * groups;
                    slot[u] = sRow[iu] * k + t;
                    a[u] = sA[iu];
                    v[u] = dH[(size_t)(uint32_t)sCol[iu] * (uint32_t)D + sIdx[slot[u]]];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) lds_add(tile + slot[u], a[u] * v[u]);
            }
            for (; i < n; i += groups) {
                const int slot = sRow[i] * k + t;
                const float v = dH[(size_t)(uint32_t)sCol[i] * (uint32_t)D + sIdx[slot]];
                lds_add(tile + slot, sA[i] * v);
            }
        }
        __syncthreads();
    }

    float* out = dXs + (size_t)r0 * k;
    const int total = nr * k;
    if (accumulate) {
        for (int i = tid; i < total; i += kThreads) out[i] += tile[i];
    } else {
        for (int i = tid; i < total; i += kThreads) out[i] = tile[i];
    }
}

int launch_spmm_bwd(const dr_csr* At, const float* dH, const uint16_t* xs_idx, int D, int k, float* dXs,
                    int accumulate, hipStream_t s) {
    const int N = (int)At->n_rows;
    int R = 2048 / k;
    if (R < 1) R = 1;
    if (R > 64) R = 64;
    const int n_tiles = (N + R - 1) / R;
    const int per_xcd = (n_tiles + kNumXcd - 1) / kNumXcd;
    int lpe_log2 = pow2_ceil_log2(k);
    if (lpe_log2 > 8) lpe_log2 = 8;
    const size_t lds = sizeof(float) * (size_t)R * k + sizeof(int) * (size_t)(R + 1 + 3 * kChunk) +
                       sizeof(uint16_t) * (size_t)R * k;
    hipLaunchKernelGGL(spmm_bwd_kernel, dim3((unsigned)(per_xcd * kNumXcd)), dim3(kThreads), lds, s, At->rowptr,
                       At->colidx, At->vals, dH, xs_idx, dXs, N, D, k, R, lpe_log2, n_tiles, per_xcd,
                       accumulate ? 1 : 0);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

}  // namespace drc
