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
    int32_t* row_start;      // [n_tiles][65]      offsets of the rows' records inside the tile (entries past the rows = records);
                             //                    every row's records are padded to a multiple of 4 with zero-valued ones
    int32_t* cols;           // [n_tiles][ccap]    distinct gathered rows (padded with a valid one)
    int2* recs;              // [n_recs]           (index of the gathered row within the tile's list, bits of the edge value)
    int device, n_cu;
};

namespace drc {

constexpr int kStRows = 64;        // rows per tile at most
constexpr int kStThreads = 1024;   // one persistent workgroup per compute unit: 4 wavefronts per SIMD
constexpr int kStEdgeCap = 2048;   // edge records per tile
constexpr int kStTileBytes = 49152;   // LDS bytes of one column slab of the tile's gathered rows
constexpr int kStUnroll = 4;       // edges per lane group and trip of the inner loop
constexpr int kStRecRegs = kStEdgeCap / kStThreads;   // records of the next tile a thread holds while the current one computes
constexpr int kStRing = 4;         // tiles whose heads (gathered rows, row ids, row offsets) are resident in LDS
constexpr int kStStartPad = kStRows + 4;

__host__ __device__ constexpr size_t staged_lds_bytes(int cw, int ccap, int ecap) {
    return sizeof(float) * (size_t)ccap * cw + 2 * sizeof(int2) * (size_t)ecap + sizeof(int2) * kStUnroll +
           sizeof(float) * kStThreads * 4 + sizeof(int) * kStRing * ((size_t)ccap + kStRows + kStStartPad + 4);
}

typedef float v4f __attribute__((ext_vector_type(4)));     // a native vector: arrays of it stay in registers
typedef int v4i __attribute__((ext_vector_type(4)));

// A persistent workgroup walks a contiguous range of tiles; the work is a stream of jobs (tile, column slab).  While it
// computes on one job, the loads of the next two are in flight in two register sets, each written to LDS after the
// barrier that ends the job still reading the old slab.  What the loads need to know of a tile -- its gathered rows,
// row ids, row offsets, record range: the tile's head -- is fetched three tiles ahead and parked in a ring of LDS
// slots; the records and saved columns of the next tile are fetched during the whole current tile.
// Which register set a job uses is a compile-time fact (NS slabs per tile, two tiles per trip of the loop): a set
// chosen at run time would have to be merged with selects, and a select needs its load to have landed.  For the
// same reason no load below is conditional: addresses are clamped to something valid and the result is ignored.
template <int CW, int KS, int NS>
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
    extern __shared__ float4 smem4[];
    float* sTile = reinterpret_cast<float*>(smem4);                              // [ccap][CW]
    long long* sRec8 = reinterpret_cast<long long*>(sTile + (size_t)ccap * CW);  // [2][ecap] records of this tile / the next
    long long* sZero = sRec8 + 2 * (size_t)ecap;                                 // [kStUnroll] records of value zero: what a lane group reads once its row has ended
    float* sScr = reinterpret_cast<float*>(sZero + kStUnroll);                   // [NQ][CW]
    int* sCols = reinterpret_cast<int*>(sScr + kStThreads * 4);                  // [kStRing][ccap]
    int* sRows = sCols + kStRing * ccap;                                         // [kStRing][kStRows]
    int* sStart = sRows + kStRing * kStRows;                                     // [kStRing][kStStartPad]
    int* sDesc = sStart + kStRing * kStStartPad;                                 // [kStRing][4] (record offset, records, gathered rows, rows)

    // Each XCD owns one contiguous range of tiles (workgroups are dealt to the XCDs round-robin) and its workgroups walk
    // it abreast: at step i the XCD's L workgroups hold L consecutive tiles -- with a placement order one compact patch
    // of the layout, whose shared dH rows the XCD's L2 fetches from memory once.
    const int L = gridDim.x / kNumXcd, xcd = blockIdx.x % kNumXcd, local = blockIdx.x / kNumXcd;
    const int x_begin = (int)((long long)xcd * n_tiles / kNumXcd), x_end = (int)((long long)(xcd + 1) * n_tiles / kNumXcd);
    const int n_my = (x_end - x_begin - local + L - 1) / L;          // tiles of this workgroup: x_begin + local + i * L
    if (n_my <= 0) return;
    const int t_begin = 0, t_end = n_my;                             // from here on a tile is named by its step i
#define DRC_TILE_ID(I) (x_begin + local + min((I), n_my - 1) * L)

    const int tid = threadIdx.x;
    const int q = tid / LPR, l = tid % LPR;
    float* scr = sScr + q * CW;
    const float* my_cols = dH + l * 4;              // this thread's 4 columns of slab 0
    const long long* recs8 = reinterpret_cast<const long long*>(recs);
    const int* desc_i = reinterpret_cast<const int*>(desc);

    int h_col, h_row, h_start, h_desc;              // a tile's head on its way to the ring
    v4f pre[2][NL];                                 // the slabs of the next two jobs
    long long nrec[kStRecRegs];                     // the next tile's records
    int ci[RPQ][KS], ci_next[RPQ][KS];              // saved columns of this thread's slots: this tile, the next

#define DRC_LOAD_HEAD(T)                                                                                      \
    do {                                                                                                      \
        const int t_ = DRC_TILE_ID(T);                                                                        \
        h_col = cols[(size_t)t_ * ccap + min(tid, ccap - 1)];                                                 \
        h_row = rows[(size_t)t_ * kStRows + min(tid, kStRows - 1)];                                           \
        h_start = row_start[(size_t)t_ * (kStRows + 1) + min(tid, kStRows)];                                  \
        h_desc = desc_i[(size_t)t_ * 4 + (tid & 3)];                                                          \
    } while (0)
#define DRC_PARK_HEAD(T)                                                                                      \
    do {                                                                                                      \
        const int s_ = (T) & (kStRing - 1);                                                                   \
        if (tid < ccap) sCols[s_ * ccap + tid] = h_col;                                                       \
        if (tid < kStRows) sRows[s_ * kStRows + tid] = h_row;                                                 \
        if (tid <= kStRows) sStart[s_ * kStStartPad + tid] = h_start;                                         \
        if (tid < 4) sDesc[s_ * 4 + tid] = h_desc;                                                            \
    } while (0)
    // this thread's pieces of slab HH of tile TT (padding pieces re-read the tile's last gathered row)
#define DRC_FETCH(SET, TT, HH)                                                                                \
    do {                                                                                                      \
        const int* c_ = sCols + (min((TT), t_end - 1) & (kStRing - 1)) * ccap;                                \
        const float* slab_ = my_cols + (size_t)(HH) * CW;                                                     \
        _Pragma("unroll") for (int u = 0; u < NL; ++u)                                                        \
            pre[SET][u] = *reinterpret_cast<const v4f*>(slab_ + (size_t)(uint32_t)c_[(u * kStThreads + tid) / LPR] * (uint32_t)D); \
    } while (0)
    // records and saved columns of tile T (rows past the tile's and slots past k read something valid that is never used)
#define DRC_LOAD_TILE_SIDE(T, CI)                                                                             \
    do {                                                                                                      \
        const int s_ = min((T), t_end - 1) & (kStRing - 1);                                                   \
        const int e0_ = sDesc[s_ * 4 + 0], ne_ = sDesc[s_ * 4 + 1];                                           \
        _Pragma("unroll") for (int j_ = 0; j_ < kStRecRegs; ++j_)                                             \
            nrec[j_] = __builtin_nontemporal_load(recs8 + e0_ + min(j_ * kStThreads + tid, max(ne_ - 1, 0)));  \
        _Pragma("unroll") for (int ri = 0; ri < RPQ; ++ri) {                                                  \
            const int lr_ = (ri & 1) ? (ri * NQ + NQ - 1 - q) : (ri * NQ + q);                                \
            const int row_ = max(sRows[s_ * kStRows + min(lr_, kStRows - 1)], 0);                             \
            _Pragma("unroll") for (int s2 = 0; s2 < KS; ++s2)                                                 \
                CI[ri][s2] = (int)__builtin_nontemporal_load(xs_idx + (size_t)row_ * k + min(l + LPR * s2, k - 1)); \
        }                                                                                                     \
    } while (0)
#define DRC_STORE_RECORDS(T, BUF)                                                                             \
    do {                                                                                                      \
        const int ne_ = sDesc[(min((T), t_end - 1) & (kStRing - 1)) * 4 + 1];                                 \
        _Pragma("unroll") for (int j_ = 0; j_ < kStRecRegs; ++j_)                                             \
            if (j_ * kStThreads + tid < ne_)                                                                  \
                sRec8[(size_t)(BUF) * ecap + j_ * kStThreads + tid] =                                         \
                    (nrec[j_] & 0xffffffff00000000LL) | (long long)((uint32_t)nrec[j_] * (uint32_t)(CW * 4));  /* index -> byte offset of the row in the slab */ \
    } while (0)

    // One tile whose first job uses register set PAR.  Job h of the tile uses set (PAR + h) & 1 and, once its slab is in
    // LDS, refills that set with the job two ahead: slab h + 2 of this tile, or slab h + 2 - NS of the next, or (NS = 1)
    // the slab of the tile after the next.
#define DRC_TILE(PAR)                                                                                         \
    do {                                                                                                      \
        const int slot = t & (kStRing - 1);                                                                   \
        const int buf = (t - t_begin) & 1;                                                                    \
        DRC_LOAD_HEAD(t + kStRing - 1);                 /* parked when this tile is done */                   \
        DRC_LOAD_TILE_SIDE(t + 1, ci_next);             /* stored when this tile is done */                   \
        const int total = sDesc[slot * 4 + 2] * LPR;                                                          \
        const long long* rec_t = sRec8 + (size_t)buf * ecap;                                                  \
        const int* start_t = sStart + slot * kStStartPad;                                                     \
        float out[RPQ][KS];                                                                                   \
        _Pragma("unroll") for (int ri = 0; ri < RPQ; ++ri)                                                    \
            _Pragma("unroll") for (int s = 0; s < KS; ++s) out[ri][s] = 0.f;                                  \
        _Pragma("unroll") for (int h = 0; h < NS; ++h) {                                                      \
            constexpr int dummy_ = 0; (void)dummy_;                                                           \
            _Pragma("unroll") for (int u = 0; u < NL; ++u)                                                    \
                if (u * kStThreads + tid < total)                                                             \
                    *reinterpret_cast<v4f*>(sTile + (size_t)(u * kStThreads + tid) * 4) = pre[((PAR) + h) & 1][u]; \
            __syncthreads();     /* the slab (and, first slab, what was parked when the tile before ended) is in LDS */ \
            DRC_FETCH(((PAR) + h) & 1, t + (h + 2) / NS, (h + 2) % NS);                                       \
            _Pragma("unroll") for (int ri = 0; ri < RPQ; ++ri) {                                              \
                const int lr = (ri & 1) ? (ri * NQ + NQ - 1 - q) : (ri * NQ + q);                             \
                int cur = start_t[min(lr, kStRows)];            /* in records; every row starts at a multiple of kStUnroll */ \
                const int end = start_t[min(lr + 1, kStRows)];                                                \
                v4f acc = {0.f, 0.f, 0.f, 0.f};                                                               \
                const char* const tile_l = reinterpret_cast<const char*>(sTile) + l * 16;                     \
                /* four records per trip, two 16-byte LDS reads; a group whose row has ended reads the zero records */ \
                const v4i* chunk = reinterpret_cast<const v4i*>(cur < end ? rec_t + cur : sZero);             \
                v4i r01 = chunk[0], r23 = chunk[1];                                                           \
                while (__any(cur < end)) {                                                                    \
                    const v4f v0 = *reinterpret_cast<const v4f*>(tile_l + (uint32_t)r01.x);                   \
                    const v4f v1 = *reinterpret_cast<const v4f*>(tile_l + (uint32_t)r01.z);                   \
                    const v4f v2 = *reinterpret_cast<const v4f*>(tile_l + (uint32_t)r23.x);                   \
                    const v4f v3 = *reinterpret_cast<const v4f*>(tile_l + (uint32_t)r23.z);                   \
                    const float w0 = __int_as_float(r01.y), w1 = __int_as_float(r01.w);                       \
                    const float w2 = __int_as_float(r23.y), w3 = __int_as_float(r23.w);                       \
                    cur += kStUnroll;                                                                         \
                    chunk = reinterpret_cast<const v4i*>(cur < end ? rec_t + cur : sZero);                    \
                    r01 = chunk[0];                                                                           \
                    r23 = chunk[1];                                                                           \
                    acc.x = fmaf(w0, v0.x, acc.x); acc.y = fmaf(w0, v0.y, acc.y); acc.z = fmaf(w0, v0.z, acc.z); acc.w = fmaf(w0, v0.w, acc.w); \
                    acc.x = fmaf(w1, v1.x, acc.x); acc.y = fmaf(w1, v1.y, acc.y); acc.z = fmaf(w1, v1.z, acc.z); acc.w = fmaf(w1, v1.w, acc.w); \
                    acc.x = fmaf(w2, v2.x, acc.x); acc.y = fmaf(w2, v2.y, acc.y); acc.z = fmaf(w2, v2.z, acc.z); acc.w = fmaf(w2, v2.w, acc.w); \
                    acc.x = fmaf(w3, v3.x, acc.x); acc.y = fmaf(w3, v3.y, acc.y); acc.z = fmaf(w3, v3.z, acc.z); acc.w = fmaf(w3, v3.w, acc.w); \
                }                                                                                             \
                /* pick the saved columns that fall into this slab (one wavefront's LDS accesses run in program order) */ \
                *reinterpret_cast<v4f*>(scr + l * 4) = acc;                                                   \
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");                                        \
                __builtin_amdgcn_wave_barrier();                                                              \
                _Pragma("unroll") for (int s = 0; s < KS; ++s) {                                              \
                    const int col = ci[ri][s];                                                                \
                    const float picked = scr[col % CW];                                                       \
                    out[ri][s] = (col / CW == h) ? picked : out[ri][s];                                       \
                }                                                                                             \
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");                                        \
                __builtin_amdgcn_wave_barrier();                                                              \
            }                                                                                                 \
            __syncthreads();      /* nobody reads the slab any more */                                        \
        }                                                                                                     \
        _Pragma("unroll") for (int ri = 0; ri < RPQ; ++ri) {                                                  \
            const int lr = (ri & 1) ? (ri * NQ + NQ - 1 - q) : (ri * NQ + q);                                 \
            const int row = lr < kStRows ? sRows[slot * kStRows + lr] : -1;                                   \
            if (row >= 0) {                                                                                   \
                float* o = dXs + (size_t)row * k;                                                             \
                _Pragma("unroll") for (int s = 0; s < KS; ++s) {                                              \
                    const int ts = l + LPR * s;                                                               \
                    if (ts < k) o[ts] = accumulate ? (o[ts] + out[ri][s]) : out[ri][s];                       \
                }                                                                                             \
            }                                                                                                 \
        }                                                                                                     \
        DRC_PARK_HEAD(t + kStRing - 1);   /* into the slot of the tile before this one, which nobody reads any more */ \
        DRC_STORE_RECORDS(t + 1, buf ^ 1);                                                                    \
        _Pragma("unroll") for (int ri = 0; ri < RPQ; ++ri)                                                    \
            _Pragma("unroll") for (int s = 0; s < KS; ++s) ci[ri][s] = ci_next[ri][s];                        \
    } while (0)

    // ---- prologue: nothing to hide behind ----
    if (tid < kStUnroll) sZero[tid] = 0;
    for (int t = t_begin; t < t_begin + kStRing - 1; ++t) {
        DRC_LOAD_HEAD(t);
        DRC_PARK_HEAD(t);
    }
    __syncthreads();
    DRC_LOAD_TILE_SIDE(t_begin, ci);
    DRC_STORE_RECORDS(t_begin, 0);
    DRC_FETCH(0, t_begin, 0);
    DRC_FETCH(1, t_begin + 1 / NS, 1 % NS);

    for (int t = t_begin; t < t_end;) {
        DRC_TILE(0);
        if (++t >= t_end) break;
        DRC_TILE(NS & 1);
        ++t;
    }
#undef DRC_TILE_ID
#undef DRC_LOAD_HEAD
#undef DRC_PARK_HEAD
#undef DRC_FETCH
#undef DRC_LOAD_TILE_SIDE
#undef DRC_STORE_RECORDS
#undef DRC_TILE
}

static int lds_limit(int* out) {
    int dev = 0, v = 0;
    DRC_HIP(hipGetDevice(&dev));
    DRC_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
    *out = v;
    return DR_OK;
}

template <int CW, int KS, int NS>
static int launch_staged(const dr_spmm_plan* p, const float* dH, const uint16_t* xs_idx, int k, float* dXs, int accumulate,
                         hipStream_t s) {
    const size_t lds = staged_lds_bytes(p->cw, p->ccap, p->ecap);
    static bool raised = false;      // per instantiation
    if (!raised) {
        DRC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&spmm_bwd_staged_kernel<CW, KS, NS>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        raised = true;
    }
    // one persistent workgroup per compute unit, a multiple of the XCD count
    int n_wg = std::min(p->n_cu, p->n_tiles);
    n_wg = (n_wg + kNumXcd - 1) / kNumXcd * kNumXcd;
    hipLaunchKernelGGL((spmm_bwd_staged_kernel<CW, KS, NS>), dim3((unsigned)n_wg), dim3(kStThreads), lds, s, p->desc, p->rows,
                       p->row_start, p->cols, p->recs, dH, xs_idx, dXs, p->D, k, p->n_tiles, p->ccap, p->ecap, accumulate ? 1 : 0);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

template <int CW, int KS>
static int launch_staged_ns(const dr_spmm_plan* p, const float* dH, const uint16_t* xs_idx, int k, float* dXs, int accumulate,
                            hipStream_t s) {
    switch (p->D / CW) {
        case 1: return launch_staged<CW, KS, 1>(p, dH, xs_idx, k, dXs, accumulate, s);
        case 2: return launch_staged<CW, KS, 2>(p, dH, xs_idx, k, dXs, accumulate, s);
        case 3: return launch_staged<CW, KS, 3>(p, dH, xs_idx, k, dXs, accumulate, s);
        case 4: return launch_staged<CW, KS, 4>(p, dH, xs_idx, k, dXs, accumulate, s);
    }
    return fail(DR_ERR_UNSUPPORTED, "dr_spmm_bwd_planned: D = %d needs more than 4 column slabs", p->D);
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
        if (ks <= 1) return launch_staged_ns<CW, 1>(p, dH, xs_idx, k, dXs, accumulate, s);          \
        if (ks <= 2) return launch_staged_ns<CW, 2>(p, dH, xs_idx, k, dXs, accumulate, s);          \
        if (ks <= 4) return launch_staged_ns<CW, 4>(p, dH, xs_idx, k, dXs, accumulate, s);          \
        if (ks <= 8) return launch_staged_ns<CW, 8>(p, dH, xs_idx, k, dXs, accumulate, s);          \
    } while (0)
    if (p->cw == 64) DRC_STAGED(64);
    else DRC_STAGED(32);
#undef DRC_STAGED
    return fail(DR_ERR_UNSUPPORTED, "dr_spmm_bwd_planned: k = %d exceeds %d for plans of D = %d", k, 8 * lpr, p->D);
}

// ---------------------------------------------------------------------------------------------------
// plan: tiles from the processing order (host side; once per relation)
// ---------------------------------------------------------------------------------------------------

static inline int pad_unroll(int deg) { return (deg + kStUnroll - 1) / kStUnroll * kStUnroll; }

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
            const bool fits = ncur + (int)fresh.size() <= ccap && ecur + pad_unroll(deg) <= ecap && rows_in < kStRows;
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
        ecur += pad_unroll(deg);
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
    std::vector<int2> recs;
    recs.reserve((size_t)E + (size_t)n * (kStUnroll - 1) / 2 + 16);
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
                recs.push_back(make_int2(ci[(size_t)q], bits));
                ++w;
            }
            // zero-valued records up to the next multiple of the inner loop's trip (they read the tile's first gathered row)
            for (; w % kStUnroll; ++w) recs.push_back(make_int2(0, 0));
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
