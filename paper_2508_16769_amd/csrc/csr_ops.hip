// Per-graph setup kernels: module edge values (mean / symmetric normalisation) and the stable CSR
// transpose used by the backward pass (paper Alg. 2, stage 1).  These run once per graph, not per
// iteration; they are written for clarity and determinism, not tuned.
#include "dr_internal.h"

#include <mutex>

namespace drc {

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

int launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t s) {
    if (n == 0) return DR_OK;
    size_t blocks = (n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, n, v);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

// row of edge e: largest i with rowptr[i] <= e (rows may be empty)
__device__ __forceinline__ int row_of_edge(const int32_t* __restrict__ rowptr, int n_rows, int e) {
    int lo = 0, hi = n_rows;  // invariant: rowptr[lo] <= e < rowptr[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (rowptr[mid] <= e) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ void count_columns_kernel(const int32_t* __restrict__ colidx, int nnz, int32_t* __restrict__ count) {
    int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < nnz) atomicAdd(&count[colidx[e]], 1);
}

__global__ void normalize_kernel(int mode, const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                                 int n_rows, int nnz, const int32_t* __restrict__ deg_out,
                                 float* __restrict__ vals) {
    int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= nnz) return;
    int i = row_of_edge(rowptr, n_rows, e);
    int di = rowptr[i + 1] - rowptr[i];
    if (mode == DR_NORM_MEAN) {
        vals[e] = (float)(1.0 / (double)di);
    } else {
        int dj = deg_out[colidx[e]];
        double a = (double)(di > 1 ? di : 1) * (double)(dj > 1 ? dj : 1);
        vals[e] = (float)(1.0 / sqrt(a));
    }
}

int launch_csr_normalize(int mode, int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t* rowptr,
                         const int32_t* colidx, float* vals_out, void* ws, hipStream_t s) {
    int32_t* deg_out = static_cast<int32_t*>(ws);
    unsigned blocks = (unsigned)((nnz + 255) / 256);
    if (mode == DR_NORM_SYM) {
        if (int rc = launch_fill_u32(reinterpret_cast<uint32_t*>(deg_out), (size_t)n_cols, 0u, s)) return rc;
        hipLaunchKernelGGL(count_columns_kernel, dim3(blocks), dim3(256), 0, s, colidx, (int)nnz, deg_out);
    }
    hipLaunchKernelGGL(normalize_kernel, dim3(blocks), dim3(256), 0, s, mode, rowptr, colidx, (int)n_rows, (int)nnz,
                       deg_out, vals_out);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

// ---------------------------------------------------------------------------------------------------
// Edge values without a workspace argument: the column counts live in a device array that is part of the
// library image.  The array's name is only a host-side handle; its device address is looked up once per
// device and that pointer is what the kernels and the fill receive.
// ---------------------------------------------------------------------------------------------------

static __device__ __align__(256) int32_t scratch[DR_NOALLOC_MAX_COLS + 64];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static int32_t* g_scratch_ptr[kMaxDevices] = {};

static int scratch_of_current_device(int32_t** out) {
    int dev = -1;
    DRC_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(DR_ERR_UNSUPPORTED, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        DRC_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (p == nullptr) return fail(DR_ERR_HIP, "hipGetSymbolAddress returned a null address for the scratch array");
        g_scratch_ptr[dev] = static_cast<int32_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return DR_OK;
}

int launch_csr_normalize_noalloc(int mode, int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t* rowptr,
                                 const int32_t* colidx, float* vals_out, hipStream_t s) {
    int32_t* deg_out = nullptr;
    if (mode == DR_NORM_SYM) DRC_TRY(scratch_of_current_device(&deg_out));   // cleared by the launcher's fill kernel
    return launch_csr_normalize(mode, n_rows, n_cols, nnz, rowptr, colidx, vals_out, deg_out, s);
}

// ---------------------------------------------------------------------------------------------------
// stable transpose
//   1. count[c+1] += 1 per stored entry (integer atomics: order does not matter)
//   2. inclusive scan -> t_rowptr
//   3. every entry e takes some slot of its column segment (atomic cursor) and records key e there
//   4. per segment, each entry's final place is the number of smaller keys in the segment: increasing e
//      is exactly "increasing original row, then storage order", so the result is the stable order
//      whatever slots step 3 handed out.  Segments of up to 16 entries are ranked inside a group of 16 lanes, up to
//      64 inside a wavefront, longer ones (high-fanout nets) by a workgroup through LDS.
// ---------------------------------------------------------------------------------------------------

constexpr int kScanBlock = 1024;

__device__ __forceinline__ int block_inclusive_scan(int v, int* smem /* [kScanBlock/64] */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    if (lane == 63) smem[wave] = x;
    __syncthreads();
    if (wave == 0) {
        int w = (lane < kScanBlock / 64) ? smem[lane] : 0;
#pragma unroll
        for (int d = 1; d < kScanBlock / 64; d <<= 1) {
            int y = __shfl_up(w, d, 64);
            if (lane >= d) w += y;
        }
        if (lane < kScanBlock / 64) smem[lane] = w;
    }
    __syncthreads();
    int prefix = (wave > 0) ? smem[wave - 1] : 0;
    __syncthreads();
    return x + prefix;
}

// a[0..n) -> per-block totals
__global__ __launch_bounds__(kScanBlock) void scan_block_sums_kernel(const int32_t* __restrict__ a, int n,
                                                                     int32_t* __restrict__ sums) {
    __shared__ int smem[kScanBlock / 64];
    int i = blockIdx.x * kScanBlock + threadIdx.x;
    int v = (i < n) ? a[i] : 0;
    int inc = block_inclusive_scan(v, smem);
    if (threadIdx.x == kScanBlock - 1) sums[blockIdx.x] = inc;
}

// exclusive scan of the block totals, one workgroup, sequential over chunks
__global__ __launch_bounds__(kScanBlock) void scan_sums_kernel(int32_t* __restrict__ sums, int nb) {
    __shared__ int smem[kScanBlock / 64];
    __shared__ int carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int base = 0; base < nb; base += kScanBlock) {
        int i = base + threadIdx.x;
        int v = (i < nb) ? sums[i] : 0;
        int inc = block_inclusive_scan(v, smem);
        int carry = carry_s;
        __syncthreads();
        if (i < nb) sums[i] = carry + inc - v;
        if (threadIdx.x == kScanBlock - 1) carry_s = carry + inc;
        __syncthreads();
    }
}

__global__ __launch_bounds__(kScanBlock) void scan_apply_kernel(int32_t* __restrict__ a, int n,
                                                                const int32_t* __restrict__ sums) {
    __shared__ int smem[kScanBlock / 64];
    int i = blockIdx.x * kScanBlock + threadIdx.x;
    int v = (i < n) ? a[i] : 0;
    int inc = block_inclusive_scan(v, smem);
    if (i < n) a[i] = inc + sums[blockIdx.x];
}

__global__ void transpose_scatter_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                                         int n_rows, int nnz, const int32_t* __restrict__ t_rowptr,
                                         int32_t* __restrict__ cursor, int32_t* __restrict__ key,
                                         int32_t* __restrict__ erow) {
    int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= nnz) return;
    erow[e] = row_of_edge(rowptr, n_rows, e);
    int c = colidx[e];
    int slot = t_rowptr[c] + atomicAdd(&cursor[c], 1);
    key[slot] = e;
}

// Step 4 for rows of up to 64 entries.  A group of 16 lanes owns one output row (four rows per wavefront): its keys
// sit in the group's registers and every entry counts the smaller keys of its row through 15 lane rotations.  Rows of
// 17 .. 64 entries are then ranked by the whole wavefront, one after the other, their keys broadcast lane by lane.
// Longer rows are only noted down (in any order: each is handled on its own by the kernel below).
__global__ __launch_bounds__(256) void transpose_place_kernel(const int32_t* __restrict__ t_rowptr, int n_cols,
                                                              const int32_t* __restrict__ key,
                                                              const int32_t* __restrict__ erow,
                                                              const float* __restrict__ vals,
                                                              int32_t* __restrict__ t_colidx,
                                                              float* __restrict__ t_vals,
                                                              int32_t* __restrict__ long_rows,
                                                              int32_t* __restrict__ n_long) {
    const int lane = threadIdx.x & 63, l = lane & 15, grp = lane >> 4;
    const int wave = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int j = wave * 4 + grp;
    const int b = j < n_cols ? t_rowptr[j] : 0;
    const int d = j < n_cols ? t_rowptr[j + 1] - b : 0;
    if (d <= 16) {
        const int my = l < d ? key[b + l] : 0x7fffffff;        // padding keys rank behind every entry
        int rank = 0;
#pragma unroll
        for (int r = 1; r < 16; ++r) rank += (__shfl(my, (l + r) & 15, 16) < my) ? 1 : 0;
        if (l < d) {
            t_colidx[b + rank] = erow[my];
            if (t_vals) t_vals[b + rank] = vals[my];
        }
    }
    // rows of this wavefront that one group cannot hold
    for (int g = 0; g < 4; ++g) {
        const int dg = __builtin_amdgcn_readfirstlane(__shfl(d, g * 16, 64));      // wave-uniform by construction
        const int bg = __builtin_amdgcn_readfirstlane(__shfl(b, g * 16, 64));
        if (dg <= 16) continue;
        if (dg > 64) {
            if (lane == 0) long_rows[atomicAdd(n_long, 1)] = wave * 4 + g;
            continue;
        }
        const int my = lane < dg ? key[bg + lane] : 0x7fffffff;
        int rank = 0;
        for (int q = 0; q < dg; ++q) rank += (__builtin_amdgcn_readlane(my, q) < my) ? 1 : 0;
        if (lane < dg) {
            t_colidx[bg + rank] = erow[my];
            if (t_vals) t_vals[bg + rank] = vals[my];
        }
    }
}

// Step 4 for the rows noted down above: one workgroup per row; the row's keys pass through LDS in chunks and every
// entry adds up, chunk by chunk, how many keys are smaller than its own.
constexpr int kLongChunk = 2048;
__global__ __launch_bounds__(256) void transpose_place_long_kernel(const int32_t* __restrict__ t_rowptr,
                                                                   const int32_t* __restrict__ long_rows,
                                                                   const int32_t* __restrict__ n_long,
                                                                   const int32_t* __restrict__ key,
                                                                   const int32_t* __restrict__ erow,
                                                                   const float* __restrict__ vals,
                                                                   int32_t* __restrict__ t_colidx,
                                                                   float* __restrict__ t_vals) {
    __shared__ int sKey[kLongChunk];
    const int total = *n_long;
    for (int i = blockIdx.x; i < total; i += gridDim.x) {
        const int j = long_rows[i];
        const int b = t_rowptr[j], d = t_rowptr[j + 1] - b;
        for (int p0 = 0; p0 < d; p0 += 256 * 4) {               // four entries per thread and pass
            int my[4], rank[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int p = p0 + u * 256 + (int)threadIdx.x;
                my[u] = p < d ? key[b + p] : 0x7fffffff;
                rank[u] = 0;
            }
            for (int c0 = 0; c0 < d; c0 += kLongChunk) {
                const int n = min(kLongChunk, d - c0);
                __syncthreads();
                for (int q = threadIdx.x; q < n; q += 256) sKey[q] = key[b + c0 + q];
                __syncthreads();
                for (int q = 0; q < n; ++q) {
                    const int kq = sKey[q];                     // every lane reads the same word: a broadcast
#pragma unroll
                    for (int u = 0; u < 4; ++u) rank[u] += (kq < my[u]) ? 1 : 0;
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int p = p0 + u * 256 + (int)threadIdx.x;
                if (p < d) {
                    t_colidx[b + rank[u]] = erow[my[u]];
                    if (t_vals) t_vals[b + rank[u]] = vals[my[u]];
                }
            }
        }
        __syncthreads();
    }
}

static size_t align256(size_t b) { return (b + 255) & ~size_t(255); }

int launch_csr_transpose(const dr_csr* A, int32_t* t_rowptr, int32_t* t_colidx, float* t_vals, void* ws,
                         hipStream_t s) {
    const int n_rows = (int)A->n_rows, n_cols = (int)A->n_cols, nnz = (int)A->nnz;
    char* w = static_cast<char*>(ws);
    int32_t* cursor = reinterpret_cast<int32_t*>(w);
    w += align256(4 * (size_t)(n_cols + 1));
    int32_t* key = reinterpret_cast<int32_t*>(w);
    w += align256(4 * (size_t)(nnz + 1));
    int32_t* erow = reinterpret_cast<int32_t*>(w);
    w += align256(4 * (size_t)(nnz + 1));
    int32_t* sums = reinterpret_cast<int32_t*>(w);
    w += align256(4 * ((size_t)(n_cols + 1) / 1024 + 2));
    int32_t* n_long = reinterpret_cast<int32_t*>(w);            // [1] (+ padding), then the rows of more than 64 entries
    int32_t* long_rows = n_long + 64;

    if (int rc = launch_fill_u32(reinterpret_cast<uint32_t*>(n_long), 1, 0u, s)) return rc;
    if (int rc = launch_fill_u32(reinterpret_cast<uint32_t*>(t_rowptr), (size_t)n_cols + 1, 0u, s)) return rc;
    if (int rc = launch_fill_u32(reinterpret_cast<uint32_t*>(cursor), (size_t)n_cols + 1, 0u, s)) return rc;
    if (nnz > 0) {
        unsigned eb = (unsigned)((nnz + 255) / 256);
        hipLaunchKernelGGL(count_columns_kernel, dim3(eb), dim3(256), 0, s, A->colidx, nnz, t_rowptr + 1);
        // inclusive scan of t_rowptr[1..n_cols]
        int nb = (n_cols + kScanBlock - 1) / kScanBlock;
        hipLaunchKernelGGL(scan_block_sums_kernel, dim3(nb), dim3(kScanBlock), 0, s, t_rowptr + 1, n_cols, sums);
        hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(kScanBlock), 0, s, sums, nb);
        hipLaunchKernelGGL(scan_apply_kernel, dim3(nb), dim3(kScanBlock), 0, s, t_rowptr + 1, n_cols, sums);
        hipLaunchKernelGGL(transpose_scatter_kernel, dim3(eb), dim3(256), 0, s, A->rowptr, A->colidx, n_rows, nnz,
                           t_rowptr, cursor, key, erow);
        unsigned pb = (unsigned)((n_cols + 15) / 16);          // 16 output rows per workgroup of four wavefronts
        hipLaunchKernelGGL(transpose_place_kernel, dim3(pb), dim3(256), 0, s, t_rowptr, n_cols, key, erow, A->vals,
                           t_colidx, t_vals, long_rows, n_long);
        hipLaunchKernelGGL(transpose_place_long_kernel, dim3(2048), dim3(256), 0, s, t_rowptr, long_rows, n_long, key, erow,
                           A->vals, t_colidx, t_vals);
    }
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

}  // namespace drc
