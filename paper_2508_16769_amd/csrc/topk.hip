// D-ReLU (paper Section 3.1): per row keep the k largest signed values, ties to the lowest column,
// survivors written in ascending column order as CBSR (vals, idx).
//
// One wavefront owns one row at a time.  Lane l holds columns l, 64+l, 128+l, ... (coalesced dword
// loads).  Values are mapped to order-preserving unsigned keys; the k-th largest key is found by a
// most-significant-bit-first search in which every step is one v_cmp per register plus a scalar
// popcount of the ballot, started below the previous row's sign and exponent bits when two probes confirm
// them, and with an early exit once a probe isolates exactly k elements; compaction
// positions come from mbcnt prefix counts of the keep-ballots, which yields ascending column order for
// free.  A row that is needed at two widths (one K per edge type) is loaded once and selected twice.
// The rank-ordered variant (largest value first; every smaller selection is a prefix, which degree-adaptive
// K relies on) stages the kept keys of a row in LDS in column order and lets every kept element count the
// keys that precede it: greater, or equal with a lower column.
#include "dr_internal.h"

namespace drc {

__device__ __forceinline__ uint32_t order_key(float v) {
    uint32_t u = __float_as_uint(v);
    u = (u == 0x80000000u) ? 0u : u;                    // -0.0 ties with +0.0
    // larger float <=> larger key; all keys > 0.  Negative values flip every bit, the others the sign bit only
    // (written without a branch: the scalar unit is what bounds this kernel).
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}

__device__ __forceinline__ int lanes_below(unsigned long long m) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

constexpr int kRowsInFlight = 4;   // rows whose loads are outstanding per wavefront

template <int EPL, bool DUAL, bool RANKED>
__global__ __launch_bounds__(256) void topk_rows_kernel(const float* __restrict__ X, int n, int D, int k,
                                                        float* __restrict__ vals, uint16_t* __restrict__ idx, int k2,
                                                        float* __restrict__ vals2, uint16_t* __restrict__ idx2) {
    extern __shared__ uint4 kept_keys4[];                     // RANKED: [4 wavefronts][k rounded up to 4] keys of the current row
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int k4 = (k + 3) >> 2;
    uint32_t* const my_keys = reinterpret_cast<uint32_t*>(kept_keys4 + wave * k4);
    const int stride = gridDim.x * (blockDim.x >> 6);        // rows between consecutive rows of one wavefront
    const int row0 = blockIdx.x * (blockDim.x >> 6) + wave;

    // loads are unconditional (row and column clamped to valid addresses): the next rows stay in flight
    // while the current one is selected
    float v[kRowsInFlight][EPL];
    auto load_row = [&](float (&dst)[EPL], int row) {
        const float* x = X + (size_t)min(row, n - 1) * D;
#pragma unroll
        for (int s = 0; s < EPL; ++s) dst[s] = __builtin_nontemporal_load(x + min(s * kWave + lane, D - 1));   // read once
    };
    uint32_t hint = 0, hint2 = 0;                             // thresholds of the previous row of this wavefront
    auto select_row = [&](const float (&val)[EPL], int row, int k, float* __restrict__ vals, uint16_t* __restrict__ idx,
                          uint32_t& t_hint) {
        uint32_t key[EPL];
#pragma unroll
        for (int s = 0; s < EPL; ++s) {
            const uint32_t real = order_key(val[s]);
            key[s] = (s * kWave + lane < D) ? real : 0u;      // padding key 0 < real keys
        }
        // T = largest threshold with count(key >= T) >= k  == the k-th largest key.  The search stops as
        // soon as a probe separates exactly k elements: then {key >= T} is already the answer, which on
        // tie-free data happens after about a dozen of the 32 bits.
        // The sign and exponent bits of T rarely change from one row to the next: probe the previous row's
        // leading nine bits first (two counts) and, if T does lie in that binade, search only below them.
        uint32_t T = 0;
        int top = 31;
        {
            // (for finite inputs a threshold never lies in the last binade; if hi did wrap to 0, c_hi would count
            // every element and the full search below would run)
            const uint32_t lo = t_hint & 0xff800000u, hi = lo + 0x00800000u;
            int c_lo = 0, c_hi = 0;
#pragma unroll
            for (int s = 0; s < EPL; ++s) {
                c_lo += __popcll(__builtin_amdgcn_ballot_w64(key[s] >= lo));
                c_hi += __popcll(__builtin_amdgcn_ballot_w64(key[s] >= hi));
            }
            if (c_lo >= k && c_hi < k) {
                T = lo;
                top = (c_lo == k) ? -1 : 22;          // exactly k at or above the binade's floor: done
            }
        }
        for (int bit = top; bit >= 0; --bit) {
            uint32_t cand = T | (1u << bit);
            int cnt = 0;
#pragma unroll
            for (int s = 0; s < EPL; ++s) cnt += __popcll(__builtin_amdgcn_ballot_w64(key[s] >= cand));
            if (cnt >= k) T = cand;
            if (cnt == k) break;
        }
        t_hint = T;
        int n_gt = 0;
#pragma unroll
        for (int s = 0; s < EPL; ++s) n_gt += __popcll(__builtin_amdgcn_ballot_w64(key[s] > T));
        const int need_eq = k - n_gt;                   // >= 1 ties to take, lowest columns first
        int kept_before = 0, eq_before = 0;
        const size_t base = (size_t)row * k;
        bool keep_s[EPL];
        int pos_s[EPL];
#pragma unroll
        for (int s = 0; s < EPL; ++s) {
            bool gt = key[s] > T;
            bool eq = key[s] == T;
            unsigned long long meq = __builtin_amdgcn_ballot_w64(eq);
            const bool tie_taken = (eq_before + lanes_below(meq)) < need_eq;     // evaluated by every lane: no branch
            const bool keep = gt || (eq && tie_taken);
            unsigned long long mk = __builtin_amdgcn_ballot_w64(keep);
            const int pos = kept_before + lanes_below(mk);     // position in ascending column order
            kept_before += __popcll(mk);
            eq_before += __popcll(meq);
            if constexpr (!RANKED) {
                if (keep) {                                    // stored at once: the predicate stays a lane mask
                    vals[base + pos] = val[s];
                    idx[base + pos] = (uint16_t)(s * kWave + lane);
                }
            } else {
                keep_s[s] = keep;
                pos_s[s] = pos;
            }
        }
        if constexpr (RANKED) {
            // One wavefront executes its LDS accesses in program order, so the reads below see the keys written here
            // and the next row's writes come after this row's reads; the fences keep the compiler from reordering.
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            if (lane < 4 * k4 - k) my_keys[k + lane] = 0u;     // padding keys: below every real key, so they never count
#pragma unroll
            for (int s = 0; s < EPL; ++s)
                if (keep_s[s]) my_keys[pos_s[s]] = key[s];
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int s = 0; s < EPL; ++s) {
                if (!keep_s[s]) continue;
                const uint32_t mine = key[s];
                const int p_me = pos_s[s];
                int rank = 0;
                for (int p4 = 0; p4 < k4; ++p4) {              // every lane reads the same 16 bytes: broadcast
                    const uint4 o = reinterpret_cast<const uint4*>(my_keys)[p4];
                    const int p = 4 * p4;
                    rank += (o.x > mine || (o.x == mine && p + 0 < p_me)) ? 1 : 0;
                    rank += (o.y > mine || (o.y == mine && p + 1 < p_me)) ? 1 : 0;
                    rank += (o.z > mine || (o.z == mine && p + 2 < p_me)) ? 1 : 0;
                    rank += (o.w > mine || (o.w == mine && p + 3 < p_me)) ? 1 : 0;
                }
                vals[base + rank] = val[s];
                idx[base + rank] = (uint16_t)(s * kWave + lane);
            }
            __builtin_amdgcn_wave_barrier();
        }
    };

#pragma unroll
    for (int i = 0; i < kRowsInFlight; ++i) load_row(v[i], row0 + i * stride);
    for (int base = row0; base < n; base += kRowsInFlight * stride) {
#pragma unroll
        for (int i = 0; i < kRowsInFlight; ++i) {
            const int row = base + i * stride;
            if (row < n) {
                select_row(v[i], row, k, vals, idx, hint);
                if constexpr (DUAL) select_row(v[i], row, k2, vals2, idx2, hint2);
            }
            load_row(v[i], row + kRowsInFlight * stride);
        }
    }
}

template <int EPL>
static void launch_epl(const float* X, int n, int D, int k, float* vals, uint16_t* idx, int k2, float* vals2,
                       uint16_t* idx2, bool ranked, hipStream_t s) {
    // Each wavefront strides over rows with four of them in flight, so it wants at least four rows (a wavefront with
    // one row pays the whole load latency for it: 20 000 rows took 15 us on 4096 workgroups, 9 us on 1250); beyond
    // 8192 workgroups (four rounds of 8 waves per SIMD) nothing is gained.  Measured on 20 k ... 1.2 M rows.
    const int waves_per_block = 4;
    long blocks = ((long)n + 4 * waves_per_block - 1) / (4 * waves_per_block);
    if (blocks > 8192) blocks = 8192;
    if (ranked)
        hipLaunchKernelGGL((topk_rows_kernel<EPL, false, true>), dim3((unsigned)blocks), dim3(256),
                           sizeof(uint4) * 4 * (size_t)((k + 3) / 4), s, X, n, D, k, vals, idx, 0, nullptr, nullptr);
    else if (vals2)
        hipLaunchKernelGGL((topk_rows_kernel<EPL, true, false>), dim3((unsigned)blocks), dim3(256), 0, s, X, n, D, k, vals, idx,
                           k2, vals2, idx2);
    else
        hipLaunchKernelGGL((topk_rows_kernel<EPL, false, false>), dim3((unsigned)blocks), dim3(256), 0, s, X, n, D, k, vals,
                           idx, 0, nullptr, nullptr);
}

static int launch_any(const float* X, int64_t n, int D, int k, float* vals, uint16_t* idx, int k2, float* vals2, uint16_t* idx2,
                      bool ranked, hipStream_t s) {
    if (n == 0) return DR_OK;
    if (D <= 64) launch_epl<1>(X, (int)n, D, k, vals, idx, k2, vals2, idx2, ranked, s);
    else if (D <= 128) launch_epl<2>(X, (int)n, D, k, vals, idx, k2, vals2, idx2, ranked, s);
    else if (D <= 256) launch_epl<4>(X, (int)n, D, k, vals, idx, k2, vals2, idx2, ranked, s);
    else if (D <= 512) launch_epl<8>(X, (int)n, D, k, vals, idx, k2, vals2, idx2, ranked, s);
    else launch_epl<16>(X, (int)n, D, k, vals, idx, k2, vals2, idx2, ranked, s);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

int launch_topk2(const float* X, int64_t n, int D, int k, float* vals, uint16_t* idx, int k2, float* vals2, uint16_t* idx2,
                 hipStream_t s) {
    return launch_any(X, n, D, k, vals, idx, k2, vals2, idx2, false, s);
}

int launch_topk(const float* X, int64_t n, int D, int k, float* vals, uint16_t* idx, hipStream_t s) {
    return launch_any(X, n, D, k, vals, idx, 0, nullptr, nullptr, false, s);
}

int launch_topk_ranked(const float* X, int64_t n, int D, int k, float* vals, uint16_t* idx, hipStream_t s) {
    return launch_any(X, n, D, k, vals, idx, 0, nullptr, nullptr, true, s);
}

}  // namespace drc
