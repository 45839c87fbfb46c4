// DR-SpMM backward with the gathered rows staged in LDS (paper Section 3.3 / Alg. 2 stage 2: the interim rows of a
// block are kept in shared memory and every edge reads them from there).
//
// The plain kernel of spmm.hip fetches one dH row through the L2 per edge.  In a relation whose rows share most of
// their neighbours with nearby rows (the geometric `near` relation: a cell's destinations lie in a small window
// around it), a compact set of source rows touches few distinct dH rows -- 64 rows of an 8 x 8 placement tile touch
// about 170 distinct rows for about 790 edges.  Here a workgroup owns such a set (a *tile*), copies the distinct
// dH rows it needs into LDS once, with coalesced row loads, and every edge then reads LDS.
//
//   * Tiles are formed once per relation (dr_spmm_plan_create) from a caller-given processing order of the rows: runs of
//     up to 64 consecutive rows of that order, cut early where the distinct gathered rows or the edge records would
//     not fit the LDS budget.  The order only decides which rows share a tile -- every result is written to its own
//     row, whatever the order -- so any permutation is valid; one in which rows that share neighbours sit next to
//     each other (cells sorted along a space-filling curve of their placement) is what makes the staging pay.
//   * LDS holds the tile's dH rows one column slab (64 columns) at a time, so a tile of 240 distinct rows takes
//     60 KB and two workgroups fit a compute unit: while one loads its slab the other computes.
//   * Within a slab a row of the tile is summed by a quarter wavefront: 16 lanes x 4 consecutive columns, one
//     ds_read_b128 per edge and lane, the whole 64-column partial row in registers.  Rows are sorted by length inside
//     the tile when the plan is made and dealt to the 16 quarter wavefronts in serpentine order, so the four quarters
//     of a wavefront walk rows of nearly equal length side by side and every quarter gets nearly the same total.
//   * After a row's last edge the quarter parks its 64 partial columns in LDS and picks the saved top-k columns that
//     fall into this slab; the compact outputs of a row stay in registers across the slabs and are written once.
//   * Every sum runs over the row's edges in storage order in one lane: results are reproducible bit for bit and equal
//     for every processing order; nothing is accumulated with atomics.
#include "dr_internal.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

struct dr_spmm_plan {
    int64_t n_rows, n_cols, nnz;
    int D, cw, ccap, ecap, n_tiles;
    double reuse;            // edges per distinct gathered row, summed over the tiles
    // device arrays; per-tile arrays are padded to a fixed stride so that a tile's entries are found from its number alone
    int4* desc;              // [n_tiles]          (offset of the tile's records, records, distinct gathered rows, rows)
    int32_t* rows;           // [n_tiles][64]      row ids, longest row first; -1 past the tile's rows
    int32_t* row_start;      // [n_tiles][65]      offsets of the rows' records inside the tile (entries past the rows = records)
    int32_t* cols;           // [n_tiles][ccap]    distinct gathered rows (padded with a valid one)
    int2* recs;              // [nnz]              (index of the gathered row within the tile's list, bits of the edge value)
    int device, n_cu;
};

namespace drc {

constexpr int kStRows = 64;        // rows per tile at most
constexpr int kStThreads = 1024;    // one workgroup per compute unit: 4 wavefronts per SIMD
constexpr int kStEdgeCap = 2048;   // edge records per tile
constexpr int kStTileBytes = 65536;   // LDS bytes of one column slab of the tile's gathered rows
constexpr int kStUnroll = 4;       // edges per lane group and trip of the inner loop
constexpr int kStRecRegs = kStEdgeCap / kStThreads;   // records of the next tile a thread holds while the current one computes

__host__ __device__ constexpr size_t staged_lds_bytes(int cw, int ccap, int ecap) {
    return sizeof(float) * (size_t)ccap * cw + sizeof(int2) * (size_t)ecap + sizeof(int) * (kStRows + 4) +
           sizeof(float) * kStThreads * 4;
}

// What a thread needs of a tile before anything of it can be fetched: found from the tile number alone.
template <int NL, int RPQ> struct TileHead {
    int4 d;            // desc
    int col[NL];       // gathered row of each of the thread's 16-byte pieces of a slab (padding repeats the last row)
    int row[RPQ];      // the rows of the thread's lane group (-1: none)
    int start;         // row_start[tid] (threads 0..64)
};

template <int NL, int RPQ, int LPR, int NQ>
__device__ __forceinline__ void load_head(TileHead<NL, RPQ>& x, int t, const int4* __restrict__ desc,
                                          const int32_t* __restrict__ rows, const int32_t* __restrict__ row_start,
                                          const int32_t* __restrict__ cols, int ccap, int tid) {
    x.d = desc[t];
#pragma unroll
    for (int u = 0; u < NL; ++u) x.col[u] = cols[(size_t)t * ccap + (u * kStThreads + tid) / LPR];
    const int q = tid / LPR;
#pragma unroll
    for (int ri = 0; ri < RPQ; ++ri) {
        const int lr = (ri & 1) ? (ri * NQ + NQ - 1 - q) : (ri * NQ + q);      // serpentine over the length-sorted rows
        x.row[ri] = lr < kStRows ? rows[(size_t)t * kStRows + lr] : -1;
    }
    x.start = row_start[(size_t)t * (kStRows + 1) + min(tid, kStRows)];
}

// All of a thread's pieces of one slab, unconditionally (padding pieces re-read the tile's last gathered row): the
// loads go out back to back and stay in flight together.
typedef float v4f __attribute__((ext_vector_type(4)));     // a native vector: arrays of it stay in registers

template <int NL>
__device__ __forceinline__ void fetch_slab(v4f (&pre)[NL], const int (&col)[NL], const float* __restrict__ slab, int D) {
#pragma unroll
    for (int u = 0; u < NL; ++u) pre[u] = *reinterpret_cast<const v4f*>(slab + (size_t)(uint32_t)col[u] * (uint32_t)D);
}

// A persistent workgroup walks a contiguous range of tiles.  While it computes on one tile, the loads of the next one
// are in flight: its head from the first slab on; its records, saved columns and first slab during the last slab of the
// tile before; every further slab during the slab before it.  Everything fetched ahead waits in registers and enters
// LDS after the barrier that ends the phase still reading the old contents.
template <int CW, int KS>
__global__ __launch_bounds__(kStThreads) void spmm_bwd_staged_kernel(
    const int4* __restrict__ desc, const int32_t* __restrict__ rows, const int32_t* __restrict__ row_start,
    const int32_t* __restrict__ cols, const int2* __restrict__ recs,
    const float* __restrict__ dH, const uint16_t* __restrict__ xs_idx, float* __restrict__ dXs,
    int D, int k, int n_tiles, int ccap, int ecap, int accumulate) {
    constexpr int LPR = CW / 4;                // lanes per row
    constexpr int NQ = kStThreads / LPR;       // rows in flight per workgroup
    constexpr int RPQ = (kStRows + NQ - 1) / NQ;   // rows of the tile per lane group (with 8 lanes per row half the groups idle)
    constexpr int NL = kStTileBytes / 16 / kStThreads;   // 16-byte pieces of a slab per thread
    static_assert(kStTileBytes % (16 * kStThreads) == 0 && kStEdgeCap % kStThreads == 0, "tile shape");
    using Head = TileHead<NL, RPQ>;
    extern __shared__ float4 smem4[];
    float* sTile = reinterpret_cast<float*>(smem4);                       // [ccap][CW]
    int2* sRec = reinterpret_cast<int2*>(sTile + (size_t)ccap * CW);      // [ecap]
    int* sRowStart = reinterpret_cast<int*>(sRec + ecap);                 // [kStRows + 1] (+3: alignment)
    float* sScr = reinterpret_cast<float*>(sRowStart + kStRows + 4);      // [NQ][CW], 16-byte aligned

    // contiguous tile ranges, and neighbouring ranges on one XCD (workgroups are dealt to the XCDs round-robin)
    const int n_wg = gridDim.x;
    const int wg = (blockIdx.x % kNumXcd) * (n_wg / kNumXcd) + blockIdx.x / kNumXcd;
    const int t_begin = (int)((long long)wg * n_tiles / n_wg), t_end = (int)((long long)(wg + 1) * n_tiles / n_wg);
    if (t_begin >= t_end) return;

    const int tid = threadIdx.x;
    const int q = tid / LPR, l = tid % LPR;
    float* scr = sScr + q * CW;
    const int n_slabs = D / CW;
    const float* my_cols = dH + l * 4;              // this thread's 4 columns of slab 0
    const long long* recs8 = reinterpret_cast<const long long*>(recs);
    long long* sRec8 = reinterpret_cast<long long*>(sRec);

    Head a, b;
    v4f pre[NL];
    long long nrec[kStRecRegs];
    int ci[RPQ][KS], ci_next[RPQ][KS];

    // ---- the first tile: nothing to hide behind ----
    load_head<NL, RPQ, LPR, NQ>(a, t_begin, desc, rows, row_start, cols, ccap, tid);
    fetch_slab<NL>(pre, a.col, my_cols, D);
#pragma unroll
    for (int j = 0; j < kStRecRegs; ++j) {
        const int e = j * kStThreads + tid;
        nrec[j] = __builtin_nontemporal_load(recs8 + a.d.x + min(e, max(a.d.y - 1, 0)));
    }
#pragma unroll
    for (int ri = 0; ri < RPQ; ++ri)
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int ts = min(l + LPR * s, k - 1);
            const int v = (int)__builtin_nontemporal_load(xs_idx + (size_t)max(a.row[ri], 0) * k + ts);
            ci[ri][s] = (a.row[ri] >= 0 && l + LPR * s < k) ? v : -1;
        }
#pragma unroll
    for (int j = 0; j < kStRecRegs; ++j) {
        const int e = j * kStThreads + tid;
        if (e < a.d.y) sRec8[e] = nrec[j];
    }
    if (tid <= kStRows) sRowStart[tid] = a.start;

    for (int t = t_begin; t < t_end; ++t) {
        const bool has_next = t + 1 < t_end;
        load_head<NL, RPQ, LPR, NQ>(b, has_next ? t + 1 : t, desc, rows, row_start, cols, ccap, tid);   // needed in the last slab
        float out[RPQ][KS];
#pragma unroll
        for (int ri = 0; ri < RPQ; ++ri)
#pragma unroll
            for (int s = 0; s < KS; ++s) out[ri][s] = 0.f;
        const int total = a.d.z * LPR;

        for (int h = 0; h < n_slabs; ++h) {
#pragma unroll
            for (int u = 0; u < NL; ++u) {
                const int p = u * kStThreads + tid;
                if (p < total) *reinterpret_cast<v4f*>(sTile + (size_t)p * 4) = pre[u];
            }
            __syncthreads();        // the slab, and (first slab) the tile's records and row offsets, are in LDS
            if (h + 1 < n_slabs) {
                fetch_slab<NL>(pre, a.col, my_cols + (size_t)(h + 1) * CW, D);
            } else if (has_next) {
                fetch_slab<NL>(pre, b.col, my_cols, D);
#pragma unroll
                for (int j = 0; j < kStRecRegs; ++j) {
                    const int e = j * kStThreads + tid;
                    nrec[j] = __builtin_nontemporal_load(recs8 + b.d.x + min(e, max(b.d.y - 1, 0)));   // read once
                }
#pragma unroll
                for (int ri = 0; ri < RPQ; ++ri)
#pragma unroll
                    for (int s = 0; s < KS; ++s) {
                        const int ts = min(l + LPR * s, k - 1);
                        const int v = (int)__builtin_nontemporal_load(xs_idx + (size_t)max(b.row[ri], 0) * k + ts);
                        ci_next[ri][s] = (b.row[ri] >= 0 && l + LPR * s < k) ? v : -1;
                    }
            }

            // ---- rows: records are read one trip ahead of the tile reads that need them ----
#pragma unroll
            for (int ri = 0; ri < RPQ; ++ri) {
                const int lr = (ri & 1) ? (ri * NQ + NQ - 1 - q) : (ri * NQ + q);
                int cur = sRowStart[min(lr, kStRows)];
                const int end = sRowStart[min(lr + 1, kStRows)];
                float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
                int2 rec[kStUnroll];
#pragma unroll
                for (int u = 0; u < kStUnroll; ++u) rec[u] = sRec[(cur + u < end) ? cur + u : 0];   // past the row: any valid record
                while (__any(cur < end)) {
                    float4 v[kStUnroll];
                    float w[kStUnroll];
#pragma unroll
                    for (int u = 0; u < kStUnroll; ++u) {
                        v[u] = *reinterpret_cast<const float4*>(sTile + rec[u].x * CW + l * 4);
                        w[u] = (cur + u < end) ? __int_as_float(rec[u].y) : 0.f;                    // ... with weight 0
                    }
                    cur += kStUnroll;
#pragma unroll
                    for (int u = 0; u < kStUnroll; ++u) rec[u] = sRec[(cur + u < end) ? cur + u : 0];
#pragma unroll
                    for (int u = 0; u < kStUnroll; ++u) {
                        acc.x = fmaf(w[u], v[u].x, acc.x);
                        acc.y = fmaf(w[u], v[u].y, acc.y);
                        acc.z = fmaf(w[u], v[u].z, acc.z);
                        acc.w = fmaf(w[u], v[u].w, acc.w);
                    }
                }
                // pick the saved columns that fall into this slab (one wavefront's LDS accesses run in program order)
                *reinterpret_cast<float4*>(scr + l * 4) = acc;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    const int col = ci[ri][s];
                    const float picked = scr[max(col, 0) % CW];
                    out[ri][s] = (col >= 0 && col / CW == h) ? picked : out[ri][s];
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
            __syncthreads();      // nobody reads the slab, the records or the row offsets any more
        }

#pragma unroll
        for (int ri = 0; ri < RPQ; ++ri) {
            if (a.row[ri] < 0) continue;
            float* o = dXs + (size_t)a.row[ri] * k;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int ts = l + LPR * s;
                if (ts < k) o[ts] = accumulate ? (o[ts] + out[ri][s]) : out[ri][s];
            }
        }
        if (has_next) {
#pragma unroll
            for (int j = 0; j < kStRecRegs; ++j) {
                const int e = j * kStThreads + tid;
                if (e < b.d.y) sRec8[e] = nrec[j];
            }
            if (tid <= kStRows) sRowStart[tid] = b.start;
        }
        a = b;
#pragma unroll
        for (int ri = 0; ri < RPQ; ++ri)
#pragma unroll
            for (int s = 0; s < KS; ++s) ci[ri][s] = ci_next[ri][s];
    }
}

static int lds_limit(int* out) {
    int dev = 0, v = 0;
    DRC_HIP(hipGetDevice(&dev));
    DRC_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
    *out = v;
    return DR_OK;
}

template <int CW, int KS>
static int launch_staged(const dr_spmm_plan* p, const float* dH, const uint16_t* xs_idx, int k, float* dXs, int accumulate,
                         hipStream_t s) {
    const size_t lds = staged_lds_bytes(p->cw, p->ccap, p->ecap);
    static bool raised = false;      // per instantiation
    if (!raised) {
        DRC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&spmm_bwd_staged_kernel<CW, KS>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        raised = true;
        if (getenv("DRC_DEBUG_OCCUPANCY")) {
            int nb = -1;
            (void)hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, reinterpret_cast<const void*>(&spmm_bwd_staged_kernel<CW, KS>), kStThreads, lds);
            fprintf(stderr, "spmm_bwd_staged_kernel<%d,%d>: %zu bytes of LDS, %d workgroups per CU\n", CW, KS, lds, nb);
        }
    }
    // one persistent workgroup per compute unit, a multiple of the XCD count
    int n_wg = std::min(p->n_cu, p->n_tiles);
    n_wg = (n_wg + kNumXcd - 1) / kNumXcd * kNumXcd;
    hipLaunchKernelGGL((spmm_bwd_staged_kernel<CW, KS>), dim3((unsigned)n_wg), dim3(kStThreads), lds, s, p->desc, p->rows,
                       p->row_start, p->cols, p->recs, dH, xs_idx, dXs, p->D, k, p->n_tiles, p->ccap, p->ecap, accumulate ? 1 : 0);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

int launch_spmm_bwd_planned(const dr_spmm_plan* p, const float* dH, const uint16_t* xs_idx, int k, float* dXs, int accumulate,
                            hipStream_t s) {
    if (p->n_rows == 0) return DR_OK;
    if (p->nnz == 0) {
        if (accumulate) return DR_OK;
        return launch_fill_u32(reinterpret_cast<uint32_t*>(dXs), (size_t)p->n_rows * k, 0u, s);
    }
    const int lpr = p->cw / 4;
    const int ks = (k + lpr - 1) / lpr;
#define DRC_STAGED(CW)                                                                              \
    do {                                                                                            \
        if (ks <= 1) return launch_staged<CW, 1>(p, dH, xs_idx, k, dXs, accumulate, s);             \
        if (ks <= 2) return launch_staged<CW, 2>(p, dH, xs_idx, k, dXs, accumulate, s);             \
        if (ks <= 4) return launch_staged<CW, 4>(p, dH, xs_idx, k, dXs, accumulate, s);             \
        if (ks <= 8) return launch_staged<CW, 8>(p, dH, xs_idx, k, dXs, accumulate, s);             \
    } while (0)
    if (p->cw == 64) DRC_STAGED(64);
    else DRC_STAGED(32);
#undef DRC_STAGED
    return fail(DR_ERR_UNSUPPORTED, "dr_spmm_bwd_planned: k = %d exceeds %d for plans of D = %d", k, 8 * lpr, p->D);
}

// ---------------------------------------------------------------------------------------------------
// plan: tiles from the processing order (host side; once per relation)
// ---------------------------------------------------------------------------------------------------

int spmm_plan_create(dr_spmm_plan** out, const dr_csr* A, const int32_t* row_order, int D, hipStream_t s) {
    *out = nullptr;
    const int cw = (D % 64 == 0) ? 64 : ((D % 32 == 0) ? 32 : 0);
    if (cw == 0) return fail(DR_ERR_UNSUPPORTED, "dr_spmm_plan_create: D = %d is not a multiple of 32", D);
    const int ccap = kStTileBytes / (cw * (int)sizeof(float));
    const int ecap = kStEdgeCap;
    int limit = 0;
    DRC_TRY(lds_limit(&limit));
    if ((size_t)limit < staged_lds_bytes(cw, ccap, ecap))
        return fail(DR_ERR_UNSUPPORTED, "dr_spmm_plan_create: the device offers %d bytes of LDS per workgroup, the staged kernel needs %zu",
                    limit, staged_lds_bytes(cw, ccap, ecap));
    const int64_t n = A->n_rows, m = A->n_cols, E = A->nnz;
    std::vector<int32_t> rp((size_t)n + 1), ci((size_t)E), ord((size_t)n);
    std::vector<float> av((size_t)E);
    DRC_HIP(hipMemcpyAsync(rp.data(), A->rowptr, sizeof(int32_t) * (n + 1), hipMemcpyDeviceToHost, s));
    if (E) {
        DRC_HIP(hipMemcpyAsync(ci.data(), A->colidx, sizeof(int32_t) * E, hipMemcpyDeviceToHost, s));
        DRC_HIP(hipMemcpyAsync(av.data(), A->vals, sizeof(float) * E, hipMemcpyDeviceToHost, s));
    }
    if (row_order && n) DRC_HIP(hipMemcpyAsync(ord.data(), row_order, sizeof(int32_t) * n, hipMemcpyDeviceToHost, s));
    DRC_HIP(hipStreamSynchronize(s));
    if (!row_order)
        for (int64_t i = 0; i < n; ++i) ord[(size_t)i] = (int32_t)i;
    {   // the order must be a permutation of the rows, the CSR well formed
        std::vector<char> seen((size_t)n, 0);
        for (int64_t i = 0; i < n; ++i) {
            const int32_t r = ord[(size_t)i];
            if (r < 0 || r >= n || seen[(size_t)r]) return fail(DR_ERR_INVALID_ARG, "dr_spmm_plan_create: row_order is not a permutation of 0..n_rows-1 (entry %lld = %d)", (long long)i, r);
            seen[(size_t)r] = 1;
        }
        if (rp[0] != 0 || rp[(size_t)n] != E) return fail(DR_ERR_INVALID_ARG, "dr_spmm_plan_create: rowptr does not span nnz");
        for (int64_t i = 0; i < n; ++i)
            if (rp[(size_t)i + 1] < rp[(size_t)i]) return fail(DR_ERR_INVALID_ARG, "dr_spmm_plan_create: rowptr decreases at row %lld", (long long)i);
        for (int64_t e = 0; e < E; ++e)
            if (ci[(size_t)e] < 0 || ci[(size_t)e] >= m) return fail(DR_ERR_INVALID_ARG, "dr_spmm_plan_create: column index %d outside [0, %lld)", ci[(size_t)e], (long long)m);
    }

    // greedy cut of the order into tiles
    std::vector<int32_t> tile_row{0}, tile_col{0}, cols;
    std::vector<int32_t> stamp((size_t)m, -1), loc((size_t)m, 0);
    cols.reserve((size_t)std::min<int64_t>(E, n * 4) + 16);
    std::vector<int32_t> fresh;
    int tid = 0, rows_in = 0, ncur = 0, ecur = 0;
    for (int64_t p = 0; p < n; ++p) {
        const int32_t r = ord[(size_t)p];
        const int deg = rp[(size_t)r + 1] - rp[(size_t)r];
        for (int attempt = 0; attempt < 2; ++attempt) {
            fresh.clear();
            for (int e = rp[(size_t)r]; e < rp[(size_t)r + 1]; ++e) {
                const int32_t c = ci[(size_t)e];
                if (stamp[(size_t)c] != tid) {
                    stamp[(size_t)c] = tid;
                    loc[(size_t)c] = ncur + (int)fresh.size();
                    fresh.push_back(c);
                }
            }
            const bool fits = ncur + (int)fresh.size() <= ccap && ecur + deg <= ecap && rows_in < kStRows;
            if (fits) break;
            for (int32_t c : fresh) stamp[(size_t)c] = -1;
            if (rows_in == 0)
                return fail(DR_ERR_UNSUPPORTED, "dr_spmm_plan_create: row %d has %d edges to %zu distinct rows; a tile holds %d edges and %d rows",
                            r, deg, fresh.size(), ecap, ccap);
            tile_row.push_back((int32_t)p);
            tile_col.push_back((int32_t)cols.size());
            ++tid;
            rows_in = ncur = ecur = 0;
        }
        cols.insert(cols.end(), fresh.begin(), fresh.end());
        ncur += (int)fresh.size();
        ecur += deg;
        ++rows_in;
        // the row's records are written below, once the tile's internal order is known; remember the local indices now
        for (int e = rp[(size_t)r]; e < rp[(size_t)r + 1]; ++e) ci[(size_t)e] = loc[(size_t)ci[(size_t)e]];   // column -> index in the tile
    }
    if (n > 0) {
        tile_row.push_back((int32_t)n);
        tile_col.push_back((int32_t)cols.size());
    }
    const int n_tiles = (int)tile_row.size() - 1;

    // inside a tile: longest row first (ties: order of arrival), the records in that order; per-tile arrays padded
    std::vector<int4> desc((size_t)n_tiles);
    std::vector<int32_t> rows_p((size_t)n_tiles * kStRows, -1), start_p((size_t)n_tiles * (kStRows + 1), 0);
    std::vector<int32_t> cols_p((size_t)n_tiles * ccap, 0);
    std::vector<int2> recs((size_t)E);
    int64_t w = 0;
    for (int t = 0; t < n_tiles; ++t) {
        auto b = ord.begin() + tile_row[(size_t)t], e = ord.begin() + tile_row[(size_t)t + 1];
        std::stable_sort(b, e, [&](int32_t x, int32_t y) { return rp[(size_t)x + 1] - rp[(size_t)x] > rp[(size_t)y + 1] - rp[(size_t)y]; });
        const int nr = tile_row[(size_t)t + 1] - tile_row[(size_t)t];
        const int nc = tile_col[(size_t)t + 1] - tile_col[(size_t)t];
        const int64_t e0 = w;
        for (int i = 0; i < nr; ++i) {
            const int32_t r = ord[(size_t)tile_row[(size_t)t] + i];
            rows_p[(size_t)t * kStRows + i] = r;
            start_p[(size_t)t * (kStRows + 1) + i] = (int32_t)(w - e0);
            for (int q = rp[(size_t)r]; q < rp[(size_t)r + 1]; ++q) {
                int bits;
                memcpy(&bits, &av[(size_t)q], 4);
                recs[(size_t)w++] = make_int2(ci[(size_t)q], bits);
            }
        }
        for (int i = nr; i <= kStRows; ++i) start_p[(size_t)t * (kStRows + 1) + i] = (int32_t)(w - e0);
        for (int i = 0; i < ccap; ++i)
            cols_p[(size_t)t * ccap + i] = nc ? cols[(size_t)tile_col[(size_t)t] + std::min(i, nc - 1)] : 0;
        desc[(size_t)t] = make_int4((int)e0, (int)(w - e0), nc, nr);
    }

    dr_spmm_plan* p = new (std::nothrow) dr_spmm_plan();
    if (!p) return fail(DR_ERR_HIP, "dr_spmm_plan_create: out of host memory");
    *p = dr_spmm_plan{};
    p->n_rows = n; p->n_cols = m; p->nnz = E; p->D = D; p->cw = cw; p->ccap = ccap; p->ecap = ecap; p->n_tiles = n_tiles;
    p->reuse = cols.empty() ? 0.0 : (double)E / (double)cols.size();
    (void)hipGetDevice(&p->device);
    if (hipDeviceGetAttribute(&p->n_cu, hipDeviceAttributeMultiprocessorCount, p->device) != hipSuccess || p->n_cu < 1) p->n_cu = 256;
    auto up = [&](auto** dst, const auto& v) -> hipError_t {
        using T = typename std::remove_const<typename std::remove_reference<decltype(v[0])>::type>::type;
        hipError_t e = hipMalloc(reinterpret_cast<void**>(dst), sizeof(T) * v.size() + 16);
        if (e != hipSuccess) return e;
        if (!v.empty()) e = hipMemcpyAsync(*dst, v.data(), sizeof(T) * v.size(), hipMemcpyHostToDevice, s);
        return e;
    };
    hipError_t e = up(&p->desc, desc);
    if (e == hipSuccess) e = up(&p->rows, rows_p);
    if (e == hipSuccess) e = up(&p->row_start, start_p);
    if (e == hipSuccess) e = up(&p->cols, cols_p);
    if (e == hipSuccess) e = up(&p->recs, recs);
    if (e == hipSuccess) e = hipStreamSynchronize(s);      // the host vectors go out of scope
    if (e != hipSuccess) {
        spmm_plan_destroy(p);
        return hip_fail(e, "dr_spmm_plan_create (device arrays)");
    }
    *out = p;
    return DR_OK;
}

void spmm_plan_destroy(dr_spmm_plan* p) {
    if (!p) return;
    void* bufs[] = {p->desc, p->rows, p->row_start, p->cols, p->recs};
    for (void* b : bufs)
        if (b) (void)hipFree(b);
    delete p;
}

}  // namespace drc

using namespace drc;

extern "C" {

int dr_spmm_plan_create(dr_spmm_plan** plan, const dr_csr* A, const int32_t* row_order, int32_t D, void* stream) {
    DRC_REQUIRE(plan != nullptr, "dr_spmm_plan_create: null plan pointer");
    *plan = nullptr;
    if (int rc = check_csr(A, "dr_spmm_plan_create: A", true)) return rc;
    DRC_REQUIRE(D >= 1, "dr_spmm_plan_create: D must be >= 1 (got %d)", D);
    if (D > DR_MAX_D) return fail(DR_ERR_UNSUPPORTED, "dr_spmm_plan_create: D = %d exceeds DR_MAX_D = %d", D, DR_MAX_D);
    DRC_REQUIRE(A->n_cols * (int64_t)D < (int64_t(1) << 32), "dr_spmm_plan_create: n_cols * D >= 2^32");
    return spmm_plan_create(plan, A, row_order, D, as_stream(stream));
}

int dr_spmm_plan_info(const dr_spmm_plan* plan, int64_t* n_tiles, double* reuse) {
    DRC_REQUIRE(plan != nullptr, "dr_spmm_plan_info: null plan");
    if (n_tiles) *n_tiles = plan->n_tiles;
    if (reuse) *reuse = plan->reuse;
    return DR_OK;
}

int dr_spmm_bwd_planned(const dr_spmm_plan* plan, const float* dH, const uint16_t* xs_idx, int32_t k, float* dXs,
                        int accumulate, void* stream) {
    DRC_REQUIRE(plan != nullptr, "dr_spmm_bwd_planned: null plan");
    DRC_REQUIRE(k >= 1 && k <= plan->D, "dr_spmm_bwd_planned: k = %d outside [1, D = %d]", k, plan->D);
    if (plan->n_rows == 0) return DR_OK;
    DRC_REQUIRE(dXs != nullptr && xs_idx != nullptr, "dr_spmm_bwd_planned: null dXs or xs_idx");
    DRC_REQUIRE(plan->nnz == 0 || dH != nullptr, "dr_spmm_bwd_planned: null dH");
    DRC_REQUIRE(aligned(dH, 16) && aligned(dXs, 4) && aligned(xs_idx, 2), "dr_spmm_bwd_planned: misaligned pointer (dH needs 16 bytes)");
    return launch_spmm_bwd_planned(plan, dH, xs_idx, k, dXs, accumulate, as_stream(stream));
}

int dr_spmm_plan_destroy(dr_spmm_plan* plan) {
    spmm_plan_destroy(plan);
    return DR_OK;
}

}  // extern "C"
