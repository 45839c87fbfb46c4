// DR-SpMM forward (paper Section 3.2 / Alg. 1) and backward (Section 3.3 / Alg. 2) for one relation.
//
// Work decomposition (both directions).  A workgroup is ONE wavefront and owns kRW consecutive CSR rows;
// there are no workgroup barriers to wait at, and the hardware dispatcher balances the (uneven) blocks.
//   * The wavefront is split into 8 groups of 8 lanes; a group owns one row at a time and walks that
//     row's edges in storage order, so 8 rows are in flight per wavefront (the wave64 counterpart of the
//     paper's "partition the warp into parts, one neighbour each") and every row sum has one fixed
//     order: results are reproducible bit for bit.
//   * The block's rows are ranked by degree, longest first, and a group that finishes a row takes the
//     next undealt one (a counter in LDS): the long rows start early, the short ones fill the gaps, and
//     the per-group totals come out balanced -- the paper's degree classes, resolved per block at run
//     time.  Which group sums a row does not change the order of that row's sum.
//   * Rows with more than kSolo edges are not given to one group: all 8 groups stride over their edges
//     into per-group partial sums that are then added in a fixed order (high-fanout nets, the tail of
//     the power-law `near` degrees).
//   * Edge records (source column, edge value) are staged into LDS in sorted-row order with independent
//     coalesced loads.  A group then consumes its rows as ONE stream of records across row boundaries,
//     so the gather pipeline never drains between rows (rows have only a handful of edges).
//   * Gathers are issued in two ping-pong batches of a few edges per group: while one batch is being
//     accumulated the other is in flight, and no load in the loop is conditional (exhausted lanes gather
//     a valid dummy row), which lets the compiler wait on exactly the older batch.  The batch depth is
//     chosen per k so that a wavefront stays within about 80 VGPRs and six wavefronts fit a SIMD: these
//     kernels wait on memory most of the time, and the number of wavefronts that can take turns matters
//     more than the depth of one wavefront's own pipeline (measured: 4 -> 6 wavefronts per SIMD, -3 %
//     of the whole layer step).
//   * Workgroup ids are remapped so each XCD walks a contiguous range of row blocks: neighbouring rows of
//     the spatially local `near` relation gather overlapping source rows, which then hit in that XCD's L2.
//
//   * Cache policy: what is read or written exactly once (the CSR records, the saved-index window, the
//     dense output rows) uses non-temporal loads and stores, so that the streams do not evict the gathered
//     rows from L2 and the memory-side cache (the forward output alone is 3-4x the gathered array); the
//     gathers themselves use the default policy.  Measured: -19 % on a random relation, -8 % on `near`.
//
// Forward.  Lane t of a group loads pairs [t*k/8, (t+1)*k/8) of the gathered source row with vector
// loads (one 128-byte line of values per source row at k = 32) and adds a*v into the group's private
// LDS row buffer with plain read-modify-write: the pairs of one source row have distinct columns and
// no other group touches the buffer, so no atomics are needed (ds_add_f32 runs at about 1/40 of the
// plain LDS rate on this chip).  A finished row goes to HBM in 128-byte segments.
//
// Backward.  Lane t of a group owns the compact outputs t, t+8, t+16, ... of its source row and keeps
// them in registers; per edge it reads dH[destination, idx[slot]] directly (the interleaved slot
// assignment keeps the 8 lanes of one load inside one 128-byte line of the dH row when 4k = D).
#include "dr_internal.h"

namespace drc {

constexpr int kLPE = 8;          // lanes per row group
constexpr int kNG = kWave / kLPE;  // groups per wavefront
constexpr int kRW = 32;          // rows per wavefront-workgroup
constexpr int kSolo = 32;        // rows with more edges are walked by all 8 groups together
constexpr int kCap = 256;        // edge records staged in LDS per pass (rows never straddle passes); 2 KB keeps
                                 // a forward workgroup below 7 KB of LDS, i.e. 23 workgroups per CU
constexpr int kStageIters = kCap / kWave;
constexpr int kBufPad = 4;       // row buffers are D + 4 words apart: group g starts 4 banks after group g-1
constexpr unsigned kValid = 0x80000000u, kLast = 0x40000000u, kRowMask = 0x0000ffffu;

struct WavePlan {
    int* sRp;      // [kRW + 1] row pointers of the block
    int* sOrder;   // [kRW]     slot -> local row; solo rows by degree, descending
    int* sStart;   // [kRW + 1] slot -> offset of the row's records in sorted-row order
    int2* sRec;    // [kCap]    staged (column, value bits) records
    int* sNext;    // [1]       next undealt slot of the current pass
    int n_solo;
    unsigned long long coop_mask, zero_mask;
};

__host__ __device__ constexpr int plan_ints() { return (kRW + 1) + kRW + (kRW + 1) + 2 + 2 /*pad*/ + 2 * kCap; }

__device__ __forceinline__ void lds_fence() { __syncthreads(); }   // one wavefront per workgroup: orders LDS traffic

__device__ __forceinline__ WavePlan make_plan(int* base, const int32_t* __restrict__ rowptr, int r0, int nr) {
    WavePlan p;
    p.sRp = base;
    p.sOrder = p.sRp + (kRW + 1);
    p.sStart = p.sOrder + kRW;
    p.sNext = p.sStart + (kRW + 1);
    int* r = p.sNext + 2;
    r += (reinterpret_cast<uintptr_t>(r) & 7) ? 1 : 0;   // 8-byte alignment for int2
    p.sRec = reinterpret_cast<int2*>(r);

    const int lane = threadIdx.x;
    const int rp_lo = rowptr[r0 + min(lane, nr)];
    const int rp_hi = rowptr[r0 + min(lane + 1, nr)];
    if (lane <= nr) p.sRp[lane] = rp_lo;
    const int deg = (lane < nr) ? (rp_hi - rp_lo) : -1;
    const bool solo = deg >= 1 && deg <= kSolo;
    p.coop_mask = __ballot(deg > kSolo);
    p.zero_mask = __ballot(deg == 0);
    p.n_solo = __popcll(__ballot(solo));
    // rank of every solo row among the solo rows: degree descending, row ascending
    const int key = solo ? deg : -1;
    int rank = 0;
#pragma unroll
    for (int j = 0; j < kRW; ++j) {
        const int kj = __shfl(key, j, kWave);
        rank += (kj > key || (kj == key && j < lane)) ? 1 : 0;
    }
    if (solo) {
        p.sOrder[rank] = lane;
        p.sStart[rank] = deg;
    }
    lds_fence();
    const int x = (lane < p.n_solo) ? p.sStart[lane] : 0;
    int incl = x;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int y = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += y;
    }
    lds_fence();
    if (lane <= p.n_solo) p.sStart[lane] = incl - x;     // exclusive prefix; entry n_solo = total
    lds_fence();
    return p;
}

// End slot of the pass that starts at slot sa: as many whole solo rows as fit kCap records (at least one).
__device__ __forceinline__ int pass_end(const WavePlan& p, int sa) {
    const int lane = threadIdx.x;
    const int base = p.sStart[sa];
    const bool fits = lane > sa && lane <= p.n_solo && p.sStart[lane] - base <= kCap;
    return sa + __popcll(__ballot(fits));
}

// Stages the records of solo slots [sa, sb) into sRec, laid out in slot order.  Every lane issues its
// loads (at most kStageIters, all independent) before the first one is consumed.
// With `ecls` (adaptive-K backward) the degree class of the edge's other end point, one byte per stored entry,
// travels in the two top bits of the staged column (columns stay below 2^30 there).
constexpr unsigned kColMask = 0x3fffffffu;
__device__ __forceinline__ int tag_class(int col, const uint8_t* __restrict__ ecls, int e) {
    return ecls ? (col | ((int)__builtin_nontemporal_load(ecls + e) << 30)) : col;
}

__device__ __forceinline__ void stage_solo(const WavePlan& p, const int32_t* __restrict__ colidx,
                                           const float* __restrict__ avals, int sa, int sb,
                                           const uint8_t* __restrict__ ecls = nullptr) {
    const int lane = threadIdx.x;
    const int base = p.sStart[sa];
    const int total = p.sStart[sb] - base;
    int2 r[kStageIters];
#pragma unroll
    for (int j = 0; j < kStageIters; ++j) {
        const int d = lane + kWave * j;
        const int dd = (d < total) ? d : 0;
        int lo = sa, hi = sb;                  // sStart[lo] - base <= dd < sStart[hi] - base
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (p.sStart[mid] - base <= dd) lo = mid; else hi = mid;
        }
        const int e = p.sRp[p.sOrder[lo]] + dd - (p.sStart[lo] - base);
        r[j] = make_int2(tag_class(__builtin_nontemporal_load(colidx + e), ecls, e),
                         __float_as_int(__builtin_nontemporal_load(avals + e)));
    }
#pragma unroll
    for (int j = 0; j < kStageIters; ++j) {
        const int d = lane + kWave * j;
        if (d < total) p.sRec[d] = r[j];
    }
}

// Stages records [c0, c0 + n) of one long row (n <= kCap, n >= 1).
__device__ __forceinline__ void stage_chunk(const WavePlan& p, const int32_t* __restrict__ colidx,
                                            const float* __restrict__ avals, int c0, int n,
                                            const uint8_t* __restrict__ ecls = nullptr) {
    const int lane = threadIdx.x;
    int2 r[kStageIters];
#pragma unroll
    for (int j = 0; j < kStageIters; ++j) {
        const int d = lane + kWave * j;
        const int e = c0 + ((d < n) ? d : 0);
        r[j] = make_int2(tag_class(__builtin_nontemporal_load(colidx + e), ecls, e),
                         __float_as_int(__builtin_nontemporal_load(avals + e)));
    }
#pragma unroll
    for (int j = 0; j < kStageIters; ++j) {
        const int d = lane + kWave * j;
        if (d < n) p.sRec[d] = r[j];
    }
}

// Record stream of one group.  Solo mode: the group takes the next undealt row of the pass whenever it
// finishes one (rows are queued by degree, longest first, so the groups finish together), and consumes
// the records of its rows one after the other across row boundaries.
// Strided mode (long rows): records g, g + 8, ... of the staged chunk, no row boundaries.
struct Stream {
    int cur, row_end, row, done;
    // Every member is assigned on every path (selects, no branches): with a member written on one side of a branch
    // only, the compiler keeps the record in scratch memory and stores through a selected address, and a scratch
    // access is a vector-memory operation -- waiting for it drains the gathers in flight.
    __device__ __forceinline__ void take_slot(const WavePlan& p, int li, int sa, int npass, int base) {
        const bool ok = li < npass;
        const int s = sa + (ok ? li : 0);
        const int c = p.sStart[s] - base, e = p.sStart[s + 1] - base, r = p.sOrder[s];
        cur = ok ? c : cur;
        row_end = ok ? e : row_end;
        row = ok ? r : row;
        done = ok ? done : 1;
    }
    __device__ __forceinline__ void next_row(const WavePlan& p, int sa, int npass, int base) {
        const int lane = threadIdx.x;
        int li = 0;
        if ((lane & (kLPE - 1)) == 0) li = atomicAdd(p.sNext, 1);
        li = __shfl(li, lane & ~(kLPE - 1), kWave);
        take_slot(p, li, sa, npass, base);
    }
    // returns the meta word of the record just taken and advances
    template <bool STRIDED>
    __device__ __forceinline__ unsigned advance(const WavePlan& p, int sa, int npass, int base) {
        unsigned m = kValid | (unsigned)row;
        if constexpr (STRIDED) {
            cur += kNG;
            if (cur >= row_end) done = 1;
        } else {
            if (++cur == row_end) {
                m |= kLast;
                next_row(p, sa, npass, base);
            }
        }
        return m;
    }
};

// ---------------------------------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------------------------------

// The pairs of one gathered CBSR row that one lane of a group handles.
//   KPL > 0: KPL consecutive pairs [t*KPL, (t+1)*KPL), vector loads (k = 8*KPL).
//   KPL < 0: the -KPL pairs t, t+8, t+16, ... with scalar loads, for every other k <= -8*KPL (the small K of the
//            optimal-K candidates among them).  Pairs past k are loaded from a clamped address and accumulated
//            into the padding words behind the row buffer, so no load or LDS access is conditional.
template <int KPL> struct Pairs {
    static constexpr int N = KPL > 0 ? KPL : -KPL;
    float v[N];
    uint16_t c[N];
    // `k`: pairs of the row that count (the row's stored width, or a prefix of it in the adaptive-K kernels).
    // PREFIX: with consecutive pairs per lane, send the pairs at or past k to the padding words as well.
    template <bool PREFIX = false>
    __device__ __forceinline__ void load(const float* __restrict__ vals, const uint16_t* __restrict__ idx, uint32_t rowbase,
                                         int t, int k, int D) {
        load_raw(vals, idx, rowbase, t, k, D);
        if constexpr (PREFIX && KPL > 0) {
#pragma unroll
            for (int u = 0; u < KPL; ++u)
                if (KPL * t + u >= k) c[u] = (uint16_t)(D + (t & (kBufPad - 1)));
        }
    }
    __device__ __forceinline__ void load_raw(const float* __restrict__ vals, const uint16_t* __restrict__ idx, uint32_t rowbase,
                                             int t, int k, int D) {
        if constexpr (KPL < 0) {
#pragma unroll
            for (int u = 0; u < N; ++u) {
                const int q = t + kLPE * u;
                const uint32_t off = rowbase + (uint32_t)min(q, k - 1);
                v[u] = vals[off];
                const uint16_t col = idx[off];
                c[u] = q < k ? col : (uint16_t)(D + (t & (kBufPad - 1)));
            }
        } else if constexpr (KPL == 1) {
            v[0] = vals[rowbase + t];
            c[0] = idx[rowbase + t];
        } else if constexpr (KPL == 2) {
            const uint32_t off = rowbase + 2 * t;
            float2 a = *reinterpret_cast<const float2*>(vals + off);
            ushort2 b = *reinterpret_cast<const ushort2*>(idx + off);
            v[0] = a.x; v[1] = a.y; c[0] = b.x; c[1] = b.y;
        } else {
            const uint32_t off = rowbase + KPL * t;
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
    // issued before the writes (lanes past k share padding words: what lands there is never read)
    __device__ __forceinline__ void accumulate(float* buf, float a) const {
        float old[N];
#pragma unroll
        for (int u = 0; u < N; ++u) old[u] = buf[c[u]];
#pragma unroll
        for (int u = 0; u < N; ++u) buf[c[u]] = fmaf(a, v[u], old[u]);
    }
};

__device__ __forceinline__ void flush_row(float* __restrict__ out, float* buf, int D, int t, int vec_store) {
    if (vec_store) {
        for (int c = t * 4; c < D; c += kLPE * 4) {
            float4 v = *reinterpret_cast<const float4*>(buf + c);
            __builtin_nontemporal_store(v.x, out + c);          // merged into one 16-byte streaming store
            __builtin_nontemporal_store(v.y, out + c + 1);
            __builtin_nontemporal_store(v.z, out + c + 2);
            __builtin_nontemporal_store(v.w, out + c + 3);
            *reinterpret_cast<float4*>(buf + c) = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    } else {
        for (int c = t; c < D; c += kLPE) {
            __builtin_nontemporal_store(buf[c], out + c);
            buf[c] = 0.0f;
        }
    }
}

template <int KPL, int EPI> struct FwdBatch {   // EPI consecutive stream records of one group, gathered
    Pairs<KPL> p[EPI];
    float a[EPI];
    unsigned meta[EPI];
};

// Degree classes of the adaptive-K variant (paper Section 3.2, Alg. 1 stage 2): a destination row with at most t1
// edges receives the k1 largest entries of each neighbour, one with at most t2 edges the k2 largest, the others k3.
struct DegreeK {
    int t1, t2, k2, k3;
    __device__ __forceinline__ int width(int deg, int k1) const { return deg <= t1 ? k1 : (deg <= t2 ? k2 : k3); }
    __device__ __forceinline__ int cls(int deg) const { return deg <= t1 ? 0 : (deg <= t2 ? 1 : 2); }
    __device__ __forceinline__ int width_of_class(int c, int k1) const { return c == 0 ? k1 : (c == 1 ? k2 : k3); }
};

template <int KPL, int EPI, bool STRIDED, bool ADAPT>
__device__ __forceinline__ void fwd_issue(FwdBatch<KPL, EPI>& b, Stream& st, const WavePlan& plan,
                                          const float* __restrict__ xs_vals, const uint16_t* __restrict__ xs_idx,
                                          int D, int k, int t, int g, int sa, int npass, int base, const DegreeK& dk) {
#pragma unroll
    for (int q = 0; q < EPI; ++q) {
        const bool valid = !st.done;
        const int2 rec = plan.sRec[valid ? st.cur : 0];
        const uint32_t col = valid ? (uint32_t)rec.x : 0u;   // exhausted lanes gather source row 0
        b.a[q] = __int_as_float(rec.y);
        int kk = k;                                          // pairs of the gathered row this destination takes
        if constexpr (ADAPT) kk = dk.width(plan.sRp[st.row + 1] - plan.sRp[st.row], k);   // a prefix of the rank order
        b.p[q].template load<ADAPT>(xs_vals, xs_idx, col * (uint32_t)k, t, kk, D);
        b.meta[q] = valid ? st.template advance<STRIDED>(plan, sa, npass, base) : 0u;
    }
}

template <int KPL, int EPI>
__device__ __forceinline__ void fwd_consume(const FwdBatch<KPL, EPI>& b, float* buf, float* __restrict__ Hblk,
                                            int D, int t, int vec_store) {
#pragma unroll
    for (int q = 0; q < EPI; ++q) {
        if (b.meta[q] & kValid) {
            b.p[q].accumulate(buf, b.a[q]);
            if (b.meta[q] & kLast) flush_row(Hblk + (size_t)(b.meta[q] & kRowMask) * D, buf, D, t, vec_store);
        }
    }
}

template <int KPL, int EPI, bool STRIDED, bool ADAPT>
__device__ __forceinline__ void fwd_run(Stream& st, const WavePlan& plan, const float* __restrict__ xs_vals,
                                        const uint16_t* __restrict__ xs_idx, float* buf, float* __restrict__ Hblk,
                                        int D, int k, int t, int g, int sa, int npass, int base, int vec_store,
                                        const DegreeK& dk) {
    if constexpr (KPL != 0) {
        FwdBatch<KPL, EPI> A, B;
        fwd_issue<KPL, EPI, STRIDED, ADAPT>(A, st, plan, xs_vals, xs_idx, D, k, t, g, sa, npass, base, dk);
        for (;;) {
            fwd_issue<KPL, EPI, STRIDED, ADAPT>(B, st, plan, xs_vals, xs_idx, D, k, t, g, sa, npass, base, dk);
            fwd_consume(A, buf, Hblk, D, t, vec_store);
            if (!__any(B.meta[0] & kValid)) break;
            fwd_issue<KPL, EPI, STRIDED, ADAPT>(A, st, plan, xs_vals, xs_idx, D, k, t, g, sa, npass, base, dk);
            fwd_consume(B, buf, Hblk, D, t, vec_store);
            if (!__any(A.meta[0] & kValid)) break;
        }
    } else {
        // k > 32 that is not 64 or 128: one record at a time, lane t takes pairs t, t+8, ... with scalar loads
        while (__any(!st.done)) {
            if (!st.done) {
                const int2 rec = plan.sRec[st.cur];
                const uint32_t rb = (uint32_t)rec.x * (uint32_t)k;
                const float a = __int_as_float(rec.y);
                for (int q = t; q < k; q += kLPE) {
                    const int c = xs_idx[rb + q];
                    buf[c] = fmaf(a, xs_vals[rb + q], buf[c]);
                }
                const unsigned m = st.template advance<STRIDED>(plan, sa, npass, base);
                if (m & kLast) flush_row(Hblk + (size_t)(m & kRowMask) * D, buf, D, t, vec_store);
            }
        }
    }
}

template <int KPL, int EPI, bool ADAPT>
__global__ __launch_bounds__(kWave) void spmm_fwd_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx, const float* __restrict__ avals,
    const float* __restrict__ xs_vals, const uint16_t* __restrict__ xs_idx, float* __restrict__ H,
    int M, int D, int k, int n_tiles, int per_xcd, int vec_store, DegreeK dk) {
    static_assert(!ADAPT || KPL != 0, "the adaptive-K forward needs a path that can mask pairs");
    extern __shared__ float4 smem4[];
    float* rowbuf = reinterpret_cast<float*>(smem4);                 // [kNG][D], 16-byte aligned
    const int tile_id = xcd_contiguous_tile(blockIdx.x, per_xcd);
    if (tile_id >= n_tiles) return;
    const int r0 = tile_id * kRW;
    const int nr = min(kRW, M - r0);
    const int lane = threadIdx.x;
    const int g = lane / kLPE, t = lane % kLPE;
    const int ldb = D + kBufPad;
    float* buf = rowbuf + g * ldb;
    float* Hblk = H + (size_t)r0 * D;

    for (int i = lane; i < kNG * ldb; i += kWave) rowbuf[i] = 0.0f;
    WavePlan plan = make_plan(reinterpret_cast<int*>(rowbuf + kNG * ldb), rowptr, r0, nr);

    // ---- rows without edges: zeros ----
    for (unsigned long long m = plan.zero_mask; m; m &= m - 1) {
        float* out = Hblk + (size_t)(__ffsll((long long)m) - 1) * D;
        for (int c = lane; c < D; c += kWave) __builtin_nontemporal_store(0.0f, out + c);
    }

    // ---- long rows: all groups stride over the row, partial sums added in a fixed order ----
    for (unsigned long long m = plan.coop_mask; m; m &= m - 1) {
        const int row = __ffsll((long long)m) - 1;
        const int e0 = plan.sRp[row], e1 = plan.sRp[row + 1];
        for (int c0 = e0; c0 < e1; c0 += kCap) {
            const int n = min(kCap, e1 - c0);
            lds_fence();
            stage_chunk(plan, colidx, avals, c0, n);
            lds_fence();
            Stream st{g, n, row, g >= n ? 1 : 0};
            fwd_run<KPL, EPI, true, ADAPT>(st, plan, xs_vals, xs_idx, buf, Hblk, D, k, t, g, 0, 0, 0, vec_store, dk);
        }
        lds_fence();
        float* out = Hblk + (size_t)row * D;
        for (int c = lane; c < D; c += kWave) {
            float s = 0.0f;
#pragma unroll
            for (int q = 0; q < kNG; ++q) {
                s += rowbuf[q * ldb + c];
                rowbuf[q * ldb + c] = 0.0f;
            }
            __builtin_nontemporal_store(s, out + c);
        }
        lds_fence();
    }

    // ---- all other rows, in passes of at most kCap staged records ----
    for (int sa = 0; sa < plan.n_solo;) {
        const int sb = pass_end(plan, sa);
        lds_fence();
        if (lane == 0) *plan.sNext = kNG;
        stage_solo(plan, colidx, avals, sa, sb);
        lds_fence();
        Stream st{0, 0, 0, 0};
        st.take_slot(plan, g, sa, sb - sa, plan.sStart[sa]);     // first 8 rows of the pass: one per group
        fwd_run<KPL, EPI, false, ADAPT>(st, plan, xs_vals, xs_idx, buf, Hblk, D, k, t, g, sa, sb - sa, plan.sStart[sa],
                                        vec_store, dk);
        sa = sb;
    }
}

int launch_spmm_fwd(const dr_csr* A, const float* xs_vals, const uint16_t* xs_idx, int D, int k, float* H,
                    hipStream_t s) {
    const int M = (int)A->n_rows;
    if (A->nnz == 0) return launch_fill_u32(reinterpret_cast<uint32_t*>(H), (size_t)M * D, 0u, s);
    const int n_tiles = (M + kRW - 1) / kRW;
    const int per_xcd = (n_tiles + kNumXcd - 1) / kNumXcd;
    const int vec_store = (D % 4 == 0 && aligned(H, 16)) ? 1 : 0;
    int kpl = 0;
    if (k % kLPE == 0) {
        const int q = k / kLPE;
        if (q == 1) kpl = 1;
        else if (q == 2 && aligned(xs_vals, 8) && aligned(xs_idx, 4)) kpl = 2;
        else if ((q == 4 || q == 8 || q == 16) && aligned(xs_vals, 16) && aligned(xs_idx, 8)) kpl = q;
    }
    if (kpl == 0 && k <= 4 * kLPE) kpl = -((k + kLPE - 1) / kLPE);   // strided scalar pairs, masked past k
    const size_t lds = sizeof(float) * (size_t)kNG * (D + kBufPad) + sizeof(int) * (size_t)plan_ints();
    dim3 grid((unsigned)(per_xcd * kNumXcd)), block(kWave);
#define DRC_LAUNCH_FWD(V, E)                                                                                              \
    hipLaunchKernelGGL((spmm_fwd_kernel<V, E, false>), grid, block, lds, s, A->rowptr, A->colidx, A->vals, xs_vals, xs_idx, \
                       H, M, D, k, n_tiles, per_xcd, vec_store, DegreeK{})
    switch (kpl) {
        case 1: DRC_LAUNCH_FWD(1, 4); break;
        case 2: DRC_LAUNCH_FWD(2, 3); break;
        case 4: DRC_LAUNCH_FWD(4, 2); break;
        case 8: DRC_LAUNCH_FWD(8, 1); break;
        case 16: DRC_LAUNCH_FWD(16, 1); break;
        case -1: DRC_LAUNCH_FWD(-1, 4); break;
        case -2: DRC_LAUNCH_FWD(-2, 3); break;
        case -3: DRC_LAUNCH_FWD(-3, 2); break;
        case -4: DRC_LAUNCH_FWD(-4, 2); break;
        default: DRC_LAUNCH_FWD(0, 1); break;
    }
#undef DRC_LAUNCH_FWD
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

int launch_spmm_fwd_adaptive(const dr_csr* A, const float* xr_vals, const uint16_t* xr_idx, int D, const dr_degree_classes* c,
                             float* H, hipStream_t s) {
    const int M = (int)A->n_rows, k = c->k1;
    if (A->nnz == 0) return launch_fill_u32(reinterpret_cast<uint32_t*>(H), (size_t)M * D, 0u, s);
    const int n_tiles = (M + kRW - 1) / kRW;
    const int per_xcd = (n_tiles + kNumXcd - 1) / kNumXcd;
    const int vec_store = (D % 4 == 0 && aligned(H, 16)) ? 1 : 0;
    const size_t lds = sizeof(float) * (size_t)kNG * (D + kBufPad) + sizeof(int) * (size_t)plan_ints();
    const DegreeK dk{c->t1, c->t2, c->k2, c->k3};
    dim3 grid((unsigned)(per_xcd * kNumXcd)), block(kWave);
#define DRC_LAUNCH_FWD_A(V, E)                                                                                            \
    hipLaunchKernelGGL((spmm_fwd_kernel<V, E, true>), grid, block, lds, s, A->rowptr, A->colidx, A->vals, xr_vals, xr_idx, \
                       H, M, D, k, n_tiles, per_xcd, vec_store, dk)
    // widths that fill the lanes evenly keep the vector loads of the uniform kernel (pairs past the destination's
    // width are redirected after the load); the others take the strided scalar pairs
    const bool vec = (k == 8) || (k == 16 && aligned(xr_vals, 8) && aligned(xr_idx, 4)) ||
                     ((k == 32 || k == 64) && aligned(xr_vals, 16) && aligned(xr_idx, 8));
    switch (vec ? k / kLPE + 100 : (k + kLPE - 1) / kLPE) {
        case 101: DRC_LAUNCH_FWD_A(1, 4); break;
        case 102: DRC_LAUNCH_FWD_A(2, 3); break;
        case 104: DRC_LAUNCH_FWD_A(4, 2); break;
        case 108: DRC_LAUNCH_FWD_A(8, 1); break;
        case 1: DRC_LAUNCH_FWD_A(-1, 4); break;
        case 2: DRC_LAUNCH_FWD_A(-2, 3); break;
        case 3: DRC_LAUNCH_FWD_A(-3, 2); break;
        case 4: DRC_LAUNCH_FWD_A(-4, 2); break;
        default: DRC_LAUNCH_FWD_A(-8, 1); break;   // k1 <= 64 (checked by the caller)
    }
#undef DRC_LAUNCH_FWD_A
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

// ---------------------------------------------------------------------------------------------------
// backward: rows are sources j (rows of A^T); lane t of the row's group owns compact slots
// s0 + t, s0 + t + 8, ... (KPL of them) in registers.  k larger than 8*KPL is covered by re-walking the
// block for the next window of slots.
// ---------------------------------------------------------------------------------------------------

template <int KPL, int EPI> struct BwdBatch {
    float v[EPI][KPL];
    float a[EPI];
    unsigned meta[EPI];
};

// saved columns of the slots lane t owns; ci[KPL] (one extra word) = column of the row's slot 0, which the
// adaptive-K kernel reads in place of the slots a destination does not take
template <int KPL>
__device__ __forceinline__ void load_ci(int (&ci)[KPL + 1], const uint16_t* sIdx, int row, int t) {
#pragma unroll
    for (int u = 0; u < KPL; ++u) ci[u] = sIdx[row * (kLPE * KPL) + t + kLPE * u];
    ci[KPL] = sIdx[row * (kLPE * KPL)];
}

constexpr unsigned kClassShift = 16;   // adaptive-K backward: degree class of the record's destination in meta bits 16-17

template <int KPL, int EPI, bool STRIDED, bool ADAPT>
__device__ __forceinline__ void bwd_issue(BwdBatch<KPL, EPI>& b, Stream& st, int (&ci)[KPL + 1], const WavePlan& plan,
                                          const uint16_t* sIdx, const float* __restrict__ dH, int D, int k, int t, int g,
                                          int sa, int npass, int base, const DegreeK& dk) {
#pragma unroll
    for (int q = 0; q < EPI; ++q) {
        const bool valid = !st.done;
        const int2 rec = plan.sRec[valid ? st.cur : 0];
        uint32_t col = valid ? (uint32_t)rec.x : 0u;
        unsigned cls = 0;
        if constexpr (ADAPT) { cls = col >> 30; col &= kColMask; }
        b.a[q] = __int_as_float(rec.y);
        const float* rowp = dH + (size_t)col * (uint32_t)D;
        if constexpr (ADAPT) {
            // slots at or past the destination's width read the column of slot 0 instead (a word the group's first
            // lane reads anyway): no load is conditional, and no further sector of the dH row is touched
            const int kq = dk.width_of_class((int)cls, k);
#pragma unroll
            for (int u = 0; u < KPL; ++u) b.v[q][u] = rowp[(t + kLPE * u < kq) ? ci[u] : ci[KPL]];
        } else {
#pragma unroll
            for (int u = 0; u < KPL; ++u) b.v[q][u] = rowp[ci[u]];
        }
        unsigned m = 0;
        if (valid) {
            m = st.template advance<STRIDED>(plan, sa, npass, base) | (cls << kClassShift);
            if (!STRIDED && (m & kLast) && !st.done) load_ci<KPL>(ci, sIdx, st.row, t);
        }
        b.meta[q] = m;
    }
}

template <int KPL, int EPI, bool ADAPT>
__device__ __forceinline__ void bwd_consume(const BwdBatch<KPL, EPI>& b, float (&acc)[KPL], float* __restrict__ Gblk,
                                            int k, int s0, int t, int accumulate, const DegreeK& dk) {
#pragma unroll
    for (int q = 0; q < EPI; ++q) {
        if (b.meta[q] & kValid) {
            if constexpr (ADAPT) {
                const int kq = dk.width_of_class((int)((b.meta[q] >> kClassShift) & 3u), k);
#pragma unroll
                for (int u = 0; u < KPL; ++u) acc[u] = fmaf(b.a[q], (t + kLPE * u < kq) ? b.v[q][u] : 0.f, acc[u]);
            } else {
#pragma unroll
                for (int u = 0; u < KPL; ++u) acc[u] = fmaf(b.a[q], b.v[q][u], acc[u]);
            }
            if (b.meta[q] & kLast) {
                float* o = Gblk + (size_t)(b.meta[q] & kRowMask) * k;
#pragma unroll
                for (int u = 0; u < KPL; ++u) {
                    const int slot = s0 + t + kLPE * u;
                    if (slot < k) o[slot] = accumulate ? (o[slot] + acc[u]) : acc[u];
                    acc[u] = 0.f;
                }
            }
        }
    }
}

template <int KPL, int EPI, bool STRIDED, bool ADAPT>
__device__ __forceinline__ void bwd_run(Stream& st, int (&ci)[KPL + 1], float (&acc)[KPL], const WavePlan& plan,
                                        const uint16_t* sIdx, const float* __restrict__ dH, float* __restrict__ Gblk,
                                        int D, int k, int s0, int t, int g, int sa, int npass, int base,
                                        int accumulate, const DegreeK& dk) {
    BwdBatch<KPL, EPI> A, B;
    bwd_issue<KPL, EPI, STRIDED, ADAPT>(A, st, ci, plan, sIdx, dH, D, k, t, g, sa, npass, base, dk);
    for (;;) {
        bwd_issue<KPL, EPI, STRIDED, ADAPT>(B, st, ci, plan, sIdx, dH, D, k, t, g, sa, npass, base, dk);
        bwd_consume<KPL, EPI, ADAPT>(A, acc, Gblk, k, s0, t, accumulate, dk);
        if (!__any(B.meta[0] & kValid)) break;
        bwd_issue<KPL, EPI, STRIDED, ADAPT>(A, st, ci, plan, sIdx, dH, D, k, t, g, sa, npass, base, dk);
        bwd_consume<KPL, EPI, ADAPT>(B, acc, Gblk, k, s0, t, accumulate, dk);
        if (!__any(A.meta[0] & kValid)) break;
    }
}

template <int KPL, int EPI, bool ADAPT>
__global__ __launch_bounds__(kWave) void spmm_bwd_kernel(
    const int32_t* __restrict__ t_rowptr, const int32_t* __restrict__ t_colidx, const float* __restrict__ t_vals,
    const float* __restrict__ dH, const uint16_t* __restrict__ xs_idx, float* __restrict__ dXs,
    int N, int D, int k, int n_tiles, int per_xcd, int accumulate, const uint8_t* __restrict__ ecls, DegreeK dk) {
    extern __shared__ float4 smem4[];
    constexpr int kWin = kLPE * KPL;                                       // compact slots per pass over the block
    float* part = reinterpret_cast<float*>(smem4);                         // [kNG][kWin] long-row partials
    uint16_t* sIdx = reinterpret_cast<uint16_t*>(part + kNG * kWin);       // [kRW][kWin] saved columns of the window
    const int tile_id = xcd_contiguous_tile(blockIdx.x, per_xcd);
    if (tile_id >= n_tiles) return;
    const int r0 = tile_id * kRW;
    const int nr = min(kRW, N - r0);
    const int lane = threadIdx.x;
    const int g = lane / kLPE, t = lane % kLPE;
    float* Gblk = dXs + (size_t)r0 * k;

    WavePlan plan = make_plan(reinterpret_cast<int*>(sIdx + kRW * kWin), t_rowptr, r0, nr);

    for (int s0 = 0; s0 < k; s0 += kWin) {
        // saved columns of this window for every row of the block (0 beyond k)
        lds_fence();
        for (int i = lane; i < nr * kWin; i += kWave) {
            const int row = i / kWin, w = i % kWin;
            sIdx[i] = (s0 + w < k) ? __builtin_nontemporal_load(xs_idx + (size_t)(r0 + row) * k + s0 + w) : (uint16_t)0;
        }
        lds_fence();

        // ---- rows without edges ----
        if (!accumulate) {
            for (unsigned long long m = plan.zero_mask; m; m &= m - 1) {
                float* o = Gblk + (size_t)(__ffsll((long long)m) - 1) * k;
                for (int w = lane; w < kWin; w += kWave)
                    if (s0 + w < k) o[s0 + w] = 0.0f;
            }
        }

        // ---- long rows ----
        for (unsigned long long m = plan.coop_mask; m; m &= m - 1) {
            const int row = __ffsll((long long)m) - 1;
            const int e0 = plan.sRp[row], e1 = plan.sRp[row + 1];
            int ci[KPL + 1];
            float acc[KPL];
            load_ci<KPL>(ci, sIdx, row, t);
#pragma unroll
            for (int u = 0; u < KPL; ++u) acc[u] = 0.f;
            for (int c0 = e0; c0 < e1; c0 += kCap) {
                const int n = min(kCap, e1 - c0);
                lds_fence();
                stage_chunk(plan, t_colidx, t_vals, c0, n, ADAPT ? ecls : nullptr);
                lds_fence();
                Stream st{g, n, row, g >= n ? 1 : 0};
                bwd_run<KPL, EPI, true, ADAPT>(st, ci, acc, plan, sIdx, dH, Gblk, D, k, s0, t, g, 0, 0, 0, accumulate, dk);
            }
#pragma unroll
            for (int u = 0; u < KPL; ++u) part[g * kWin + t + kLPE * u] = acc[u];
            lds_fence();
            for (int w = lane; w < kWin; w += kWave) {
                if (s0 + w < k) {
                    float s = 0.f;
#pragma unroll
                    for (int q = 0; q < kNG; ++q) s += part[q * kWin + w];
                    float* o = Gblk + (size_t)row * k + s0 + w;
                    *o = accumulate ? (*o + s) : s;
                }
            }
            lds_fence();
        }

        // ---- all other rows ----
        for (int sa = 0; sa < plan.n_solo;) {
            const int sb = pass_end(plan, sa);
            lds_fence();
            if (lane == 0) *plan.sNext = kNG;
            stage_solo(plan, t_colidx, t_vals, sa, sb, ADAPT ? ecls : nullptr);
            lds_fence();
            Stream st{0, 0, 0, 0};
            st.take_slot(plan, g, sa, sb - sa, plan.sStart[sa]);
            int ci[KPL + 1];
            float acc[KPL];
            ci[KPL] = 0;
#pragma unroll
            for (int u = 0; u < KPL; ++u) { ci[u] = 0; acc[u] = 0.f; }
            if (!st.done) load_ci<KPL>(ci, sIdx, st.row, t);
            bwd_run<KPL, EPI, false, ADAPT>(st, ci, acc, plan, sIdx, dH, Gblk, D, k, s0, t, g, sa, sb - sa, plan.sStart[sa],
                                            accumulate, dk);
            sa = sb;
        }
    }
}

static int launch_bwd_any(const dr_csr* At, const float* dH, const uint16_t* xs_idx, int D, int k, float* dXs, int accumulate,
                          const uint8_t* ecls, DegreeK dk, hipStream_t s) {
    const int N = (int)At->n_rows;
    if (At->nnz == 0) {
        if (accumulate) return DR_OK;
        return launch_fill_u32(reinterpret_cast<uint32_t*>(dXs), (size_t)N * k, 0u, s);
    }
    const int n_tiles = (N + kRW - 1) / kRW;
    const int per_xcd = (n_tiles + kNumXcd - 1) / kNumXcd;
    int kpl = 8;
    if (k <= 8) kpl = 1;
    else if (k <= 16) kpl = 2;
    else if (k <= 32) kpl = 4;
    dim3 grid((unsigned)(per_xcd * kNumXcd)), block(kWave);
    const size_t lds = sizeof(float) * (size_t)kNG * (kLPE * kpl) + sizeof(uint16_t) * (size_t)kRW * (kLPE * kpl) +
                       sizeof(int) * (size_t)plan_ints();
#define DRC_LAUNCH_BWD(V, E, A)                                                                                            \
    hipLaunchKernelGGL((spmm_bwd_kernel<V, E, A>), grid, block, lds, s, At->rowptr, At->colidx, At->vals, dH, xs_idx, dXs, \
                       N, D, k, n_tiles, per_xcd, accumulate ? 1 : 0, ecls, dk)
    if (ecls) {
        switch (kpl) {
            case 1: DRC_LAUNCH_BWD(1, 4, true); break;
            case 2: DRC_LAUNCH_BWD(2, 4, true); break;
            case 4: DRC_LAUNCH_BWD(4, 2, true); break;
            default: DRC_LAUNCH_BWD(8, 1, true); break;   // k <= 64: one window of slots (checked by the caller)
        }
    } else {
        switch (kpl) {
            case 1: DRC_LAUNCH_BWD(1, 4, false); break;
            case 2: DRC_LAUNCH_BWD(2, 4, false); break;
            case 4: DRC_LAUNCH_BWD(4, 2, false); break;
            default: DRC_LAUNCH_BWD(8, 1, false); break;
        }
    }
#undef DRC_LAUNCH_BWD
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

int launch_spmm_bwd(const dr_csr* At, const float* dH, const uint16_t* xs_idx, int D, int k, float* dXs,
                    int accumulate, hipStream_t s) {
    return launch_bwd_any(At, dH, xs_idx, D, k, dXs, accumulate, nullptr, DegreeK{}, s);
}

int launch_spmm_bwd_adaptive(const dr_csr* At, const uint8_t* edge_class, const float* dH, const uint16_t* xr_idx, int D,
                             const dr_degree_classes* c, float* dXr, int accumulate, hipStream_t s) {
    return launch_bwd_any(At, dH, xr_idx, D, c->k1, dXr, accumulate, edge_class, DegreeK{c->t1, c->t2, c->k2, c->k3}, s);
}

// class (0 low, 1 medium, 2 high) of the destination of every stored entry of At, from the forward row pointers
__global__ __launch_bounds__(256) void edge_class_kernel(const int32_t* __restrict__ t_colidx, int nnz,
                                                         const int32_t* __restrict__ a_rowptr, int t1, int t2,
                                                         uint8_t* __restrict__ out) {
    for (int e = blockIdx.x * 256 + threadIdx.x; e < nnz; e += gridDim.x * 256) {
        const int i = t_colidx[e];
        const int deg = a_rowptr[i + 1] - a_rowptr[i];
        out[e] = (uint8_t)(deg <= t1 ? 0 : (deg <= t2 ? 1 : 2));
    }
}

int launch_edge_classes(const dr_csr* At, const int32_t* a_rowptr, const dr_degree_classes* c, uint8_t* out, hipStream_t s) {
    if (At->nnz == 0) return DR_OK;
    unsigned blocks = (unsigned)((At->nnz + 255) / 256);
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(edge_class_kernel, dim3(blocks), dim3(256), 0, s, At->colidx, (int)At->nnz, a_rowptr, c->t1, c->t2, out);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

}  // namespace drc
