// Multi-layer training step (paper Section 4.1): L stacked HeteroConv layers with ReLU between them, a
// per-cell read-out pred = X_cell^(L) . w_head, mean-squared error over all cells of the batch, Adam with
// the L2 form of weight decay.  The sub-graphs of a batch are independent (Section 3.4): each runs its
// whole forward and backward on its own stream (the relation streams of its layer context fork below
// that), and the streams are joined only before the parameter update.
//
// What is new here next to the layer is element-wise or a small reduction:
//   (the ReLU between layers and its gate are folded into the layer kernels that write Y and dX)
//   head_fwd_kernel                    one wavefront per cell: dot product, residual, loss partials
//   head_bwd_kernel                    dY = dpred (x) w_head, per-workgroup partials of dw_head = Y^T dpred
//   loss_reduce_kernel, adam_kernel    fixed-order sums over sub-graphs and partials, then the update
// Every sum has a fixed order, so a step is reproducible bit for bit.
//
// Batched mode (hgnn_create_batched): the sub-graphs are stacked into ONE block-diagonal graph on the device
// (rows and columns of sub-graph q shifted by the node counts of the sub-graphs before it) and the step runs
// as a single-graph step: one launch per kernel for the whole batch instead of one per sub-graph.  A
// 20 000-cell launch fills a fraction of the chip and a streamed step of 8 x 3 layers issues some 800 of
// them, so for small sub-graphs stacking is the faster mapping of "independent sub-graphs" (Section 3.4).
#include "dr_internal.h"

#include <cmath>
#include <condition_variable>
#include <functional>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

namespace drc {

// workgroups (= partial sums) of the read-out kernels for a state of n cells: about 256 rows each, at least 64
inline int head_blocks(int64_t n) {
    int64_t b = (n + 255) / 256;
    return (int)(b < 64 ? 64 : (b > 2048 ? 2048 : b));
}
constexpr int kMaxWorkers = 8;    // host threads that enqueue sub-graphs side by side

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
    return v;
}

// pred[i] = Y[i,:] . w;  dpred[i] = scale * (pred[i] - target[i]);  loss_part[block] = sum of squared residuals
__global__ __launch_bounds__(256) void head_fwd_kernel(const float* __restrict__ Y, const float* __restrict__ w,
                                                       const float* __restrict__ target, int n, int D, float scale,
                                                       float* __restrict__ pred, float* __restrict__ dpred,
                                                       float* __restrict__ loss_part) {
    __shared__ float sq[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float acc = 0.f;                                            // squared residuals seen by this wavefront (lane 0)
    for (int row = blockIdx.x * 4 + wave; row < n; row += gridDim.x * 4) {
        float s = 0.f;
        for (int c = lane; c < D; c += kWave) s += Y[(size_t)row * D + c] * w[c];
        s = wave_sum(s);
        const float r = s - target[row];
        if (lane == 0) {
            pred[row] = s;
            dpred[row] = scale * r;
            acc += r * r;
        }
    }
    if (lane == 0) sq[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) loss_part[blockIdx.x] = (sq[0] + sq[1]) + (sq[2] + sq[3]);
}

// dY[i,c] = dpred[i] * w[c];  dw_part[block][c] = sum over the block's rows of dpred[i] * Y[i,c]
__global__ __launch_bounds__(256) void head_bwd_kernel(const float* __restrict__ Y, const float* __restrict__ w,
                                                       const float* __restrict__ dpred, int n, int D,
                                                       float* __restrict__ dY, float* __restrict__ dw_part) {
    extern __shared__ float part[];                             // [256]
    const int rows_per_pass = 256 / D;                          // D in {32,64,96,128}: 8, 4, 2, 2 row lanes
    const int c = threadIdx.x % D, rl = threadIdx.x / D;
    const bool active = rl < rows_per_pass;
    const int per_block = (n + gridDim.x - 1) / gridDim.x;
    const int r0 = blockIdx.x * per_block, r1 = min(n, r0 + per_block);
    float acc = 0.f;
    if (active) {
        const float wc = w[c];
        for (int row = r0 + rl; row < r1; row += rows_per_pass) {
            const float g = dpred[row];
            acc = fmaf(g, Y[(size_t)row * D + c], acc);
            dY[(size_t)row * D + c] = g * wc;
        }
    }
    part[threadIdx.x] = active ? acc : 0.f;
    __syncthreads();
    if (threadIdx.x < D) {
        float s = 0.f;
        for (int q = 0; q < rows_per_pass; ++q) s += part[q * D + threadIdx.x];
        dw_part[(size_t)blockIdx.x * D + threadIdx.x] = s;
    }
}

__global__ __launch_bounds__(64) void loss_reduce_kernel(const float* __restrict__ loss_part, int n_parts, float inv_n,
                                                         float* __restrict__ loss_out) {
    float s = 0.f;
    for (int i = threadIdx.x; i < n_parts; i += kWave) s += loss_part[i];
    s = wave_sum(s);
    if (threadIdx.x == 0) *loss_out = s * inv_n;
}

// dwh[c] = sum over all read-out partials (fixed order: thread t takes partials t, t + 256, ..., then a tree over
// the 256 thread sums); one workgroup per column
__global__ __launch_bounds__(256) void head_reduce_kernel(const float* __restrict__ dwh_part, int n_parts, int D,
                                                          float* __restrict__ dwh) {
    __shared__ float sh[256];
    const int c = blockIdx.x;
    float s = 0.f;
    for (int q = threadIdx.x; q < n_parts; q += 256) s += dwh_part[(size_t)q * D + c];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) dwh[c] = sh[0];
}

// g = sum over sub-graphs (fixed order) of the gradient pieces; Adam with L2 weight decay, bias-corrected
__global__ __launch_bounds__(256) void adam_kernel(float* __restrict__ theta, float* __restrict__ m, float* __restrict__ v,
                                                   float* __restrict__ grad_out, const float* __restrict__ gall,
                                                   const float* __restrict__ dwh, int n_graphs, int64_t PL, int D,
                                                   float lr, float beta1, float beta2, float omb1, float omb2,
                                                   float eps, float wd, float inv_bc1, float inv_bc2) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= PL + D) return;
    float g = 0.f;
    if (e < PL) {
        for (int q = 0; q < n_graphs; ++q) g += gall[(size_t)q * PL + e];
    } else {
        g = dwh[e - PL];
    }
    grad_out[e] = g;
    const float th = theta[e];
    g = fmaf(wd, th, g);
    const float m2 = beta1 * m[e] + omb1 * g;        // omb = 1 - beta, formed in double on the host
    const float v2 = beta2 * v[e] + omb2 * g * g;
    m[e] = m2;
    v[e] = v2;
    theta[e] = th - lr * (m2 * inv_bc1) / (sqrtf(v2 * inv_bc2) + eps);
}

// block-diagonal stacking of CSR parts: part q's rows go to [row_off, row_off + n_rows), its columns are
// shifted by col_off and its edges go to [nnz_off, nnz_off + nnz)
__global__ __launch_bounds__(256) void concat_csr_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                                                         const float* __restrict__ vals, int n_rows, int nnz, int row_off,
                                                         int col_off, int nnz_off, int write_end, int32_t* __restrict__ o_rowptr,
                                                         int32_t* __restrict__ o_colidx, float* __restrict__ o_vals) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n_rows) o_rowptr[row_off + i] = rowptr[i] + nnz_off;
    if (i == 0 && write_end) o_rowptr[row_off + n_rows] = nnz_off + nnz;
    for (int e = i; e < nnz; e += gridDim.x * 256) {
        o_colidx[nnz_off + e] = colidx[e] + col_off;
        o_vals[nnz_off + e] = vals[e];
    }
}

// up to kGatherParts row blocks, each contiguous on its own, copied behind one another (dwords)
constexpr int kGatherParts = 32;
struct GatherArgs {
    const uint32_t* src[kGatherParts];
    unsigned long long start[kGatherParts + 1];   // dword offset of part i in dst; start[n] = total
    int n;
};
__global__ __launch_bounds__(256) void gather_parts_kernel(GatherArgs a, uint32_t* __restrict__ dst) {
    const unsigned long long total = a.start[a.n];
    for (unsigned long long i = (unsigned long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (unsigned long long)gridDim.x * 256) {
        int q = 0;
        while (q + 1 < a.n && a.start[q + 1] <= i) ++q;
        dst[i] = a.src[q][i - a.start[q]];
    }
}

struct GraphState {
    dr_heteroconv* ctx;
    int64_t Nc, Nn;
    std::vector<float*> act_c, act_n;          // [L] layer outputs
    std::vector<dr_heteroconv_saved> saved;    // [L]
    std::vector<float*> G_c, G_n;              // [L+1] gradients: G[l] = dX of layer l = (after the gate) dY of layer l-1
    float* gvec;                               // this sub-graph's layer-weight gradients, theta layout (slice of gall)
    float *pred, *dpred;
    float *loss_part, *dwh_part;               // slices of the model's partial arrays
    int hb;                                    // workgroups of the read-out kernels = partials in those slices
    hipStream_t stream;
    hipEvent_t done;
    const float *X_cell, *X_net;               // caller's inputs of the last step (for inspection)
};

}  // namespace drc

namespace drc {
// Host threads that enqueue the sub-graphs of a step side by side.  They are started once, with the model, and sleep
// between steps: starting and joining threads on every step costs more than enqueueing a small sub-graph.
class EnqueuePool {
  public:
    EnqueuePool(int n_threads, int device) : rcs_(n_threads, DR_OK), errs_(n_threads) {
        for (int w = 0; w < n_threads; ++w)
            threads_.emplace_back([this, w, device]() {
                const bool dev_ok = hipSetDevice(device) == hipSuccess;
                unsigned long long seen = 0;
                for (;;) {
                    std::unique_lock<std::mutex> lock(mu_);
                    wake_.wait(lock, [&] { return stop_ || generation_ != seen; });
                    if (stop_) return;
                    seen = generation_;
                    lock.unlock();
                    int rc = DR_OK;
                    if (!dev_ok) { rc = DR_ERR_HIP; errs_[w] = "hipSetDevice failed in a worker thread"; }
                    for (int q = w; q < n_items_ && rc == DR_OK; q += (int)threads_.size()) {
                        rc = (*job_)(q);
                        if (rc != DR_OK) errs_[w] = dr_last_error();     // the error text is per thread: hand it over
                    }
                    rcs_[w] = rc;
                    lock.lock();
                    if (--pending_ == 0) done_.notify_all();
                }
            });
    }
    ~EnqueuePool() {
        {
            std::lock_guard<std::mutex> lock(mu_);
            stop_ = true;
        }
        wake_.notify_all();
        for (auto& t : threads_) t.join();
    }
    // Runs job(q) for q = 0 .. n_items-1, item q on thread q % n_threads, and waits for all of them.  Returns the first
    // failing status (with its message in *err) after every thread has finished its items.
    int run(int n_items, const std::function<int(int)>& job, std::string* err) {
        {
            std::lock_guard<std::mutex> lock(mu_);
            job_ = &job;
            n_items_ = n_items;
            pending_ = (int)threads_.size();
            ++generation_;
        }
        wake_.notify_all();
        std::unique_lock<std::mutex> lock(mu_);
        done_.wait(lock, [&] { return pending_ == 0; });
        for (size_t w = 0; w < rcs_.size(); ++w)
            if (rcs_[w] != DR_OK) { *err = errs_[w]; return rcs_[w]; }
        return DR_OK;
    }

  private:
    std::vector<std::thread> threads_;
    std::mutex mu_;
    std::condition_variable wake_, done_;
    const std::function<int(int)>* job_ = nullptr;
    int n_items_ = 0, pending_ = 0;
    unsigned long long generation_ = 0;
    bool stop_ = false;
    std::vector<int> rcs_;
    std::vector<std::string> errs_;
};

}  // namespace drc

struct dr_hgnn {
    int n_graphs, L, D;                        // n_graphs: states that are stepped (1 for a batched model)
    int n_user;                                // sub-graphs the caller sees
    bool batched;
    bool inspect;                              // also compute what training does not need: dX of the first layer, Y_net of the last
    std::vector<int64_t> off_c, off_n;         // [n_user + 1] first cell / net row of sub-graph q in the stacked graph
    std::vector<const float*> ux_c, ux_n;      // [n_user] caller's inputs of the last step (for inspection)
    dr_heteroconv* big;                        // batched: context of the stacked graph (owned)
    dr_csr big_rel[3];                         // batched: its relations (arrays in `owned`)
    float *Xc_all, *Xn_all, *tg_all;           // batched: staging for inputs the caller does not hold contiguously
    int64_t PL;                                // layer parameters: L*5*D*D
    int64_t n_cells_total;
    std::vector<drc::GraphState> g;
    std::vector<void*> owned;
    float *gall, *loss_part, *dwh_part, *dwh;  // dwh[D]: the read-out weight gradient, summed over all partials
    int n_head_parts;                          // read-out partials of all states together
    hipEvent_t fork;
    int device;
    drc::EnqueuePool* pool;                    // more than one state: the threads that enqueue them side by side
};

using namespace drc;

namespace {

int model_alloc(dr_hgnn* m, void** p, size_t bytes) {
    *p = nullptr;
    if (bytes == 0) bytes = 256;
    DRC_HIP(hipMalloc(p, bytes));
    m->owned.push_back(*p);
    return DR_OK;
}

void model_release(dr_hgnn* m) {
    if (!m) return;
    delete m->pool;
    for (void* p : m->owned) (void)hipFree(p);
    for (auto& gs : m->g) {
        if (gs.stream) (void)hipStreamDestroy(gs.stream);
        if (gs.done) (void)hipEventDestroy(gs.done);
    }
    if (m->fork) (void)hipEventDestroy(m->fork);
    if (m->big) (void)heteroconv_destroy(m->big);
    delete m;
}

template <typename T>
int alloc_t(dr_hgnn* m, T** p, size_t count) { return model_alloc(m, reinterpret_cast<void**>(p), count * sizeof(T)); }

dr_heteroconv_weights layer_weights(const float* theta, int l, int D) {
    const float* b = theta + (size_t)l * 5 * D * D;
    const size_t dd = (size_t)D * D;
    return dr_heteroconv_weights{b, b + dd, b + 2 * dd, b + 3 * dd, b + 4 * dd};
}

dr_heteroconv_wgrads layer_wgrads(float* gvec, int l, int D) {
    float* b = gvec + (size_t)l * 5 * D * D;
    const size_t dd = (size_t)D * D;
    return dr_heteroconv_wgrads{b, b + dd, b + 2 * dd, b + 3 * dd, b + 4 * dd};
}

}  // namespace

extern "C" {

int64_t hgnn_num_params(int32_t n_layers, int32_t D) {
    if (n_layers < 1 || D < 1) return 0;
    return (int64_t)n_layers * 5 * D * D + D;
}

static int create_model(dr_hgnn** model, int32_t n_graphs, dr_heteroconv* const* graphs, int32_t n_layers, bool batched) {
    DRC_REQUIRE(model != nullptr, "hgnn_create: null model");
    *model = nullptr;
    DRC_REQUIRE(n_graphs >= 1 && n_graphs <= 1024, "hgnn_create: n_graphs = %d out of range [1, 1024]", n_graphs);
    DRC_REQUIRE(n_layers >= 1 && n_layers <= 16, "hgnn_create: n_layers = %d out of range [1, 16]", n_layers);
    DRC_REQUIRE(graphs != nullptr, "hgnn_create: null graphs");
    for (int q = 0; q < n_graphs; ++q) DRC_REQUIRE(graphs[q] != nullptr, "hgnn_create: graph %d is null", q);
    for (int q = 0; q < n_graphs; ++q)
        for (int r = 0; r < q; ++r)
            DRC_REQUIRE(batched || graphs[q] != graphs[r], "hgnn_create: graphs %d and %d share one context (its scratch is per step)", r, q);
    const HeteroDims d0 = heteroconv_dims(graphs[0]);
    for (int q = 1; q < n_graphs; ++q) {   // the parameters are shared, so the width is; each sub-graph keeps its own K
        const HeteroDims d = heteroconv_dims(graphs[q]);
        DRC_REQUIRE(d.D == d0.D, "hgnn_create: graph %d has D = %d, graph 0 has %d", q, d.D, d0.D);
        DRC_REQUIRE(!batched || (d.k_near == d0.k_near && d.k_pins == d0.k_pins && d.k_self == d0.k_self && d.k_pinned == d0.k_pinned),
                    "hgnn_create_batched: graph %d has other K than graph 0 (one launch serves the whole batch)", q);
    }
    dr_hgnn* m = new (std::nothrow) dr_hgnn();
    if (!m) return fail(DR_ERR_HIP, "hgnn_create: out of host memory");
    m->n_user = n_graphs; m->batched = batched; m->inspect = false;
    m->n_graphs = batched ? 1 : n_graphs; m->L = n_layers; m->D = d0.D;
    m->PL = (int64_t)n_layers * 5 * d0.D * d0.D;
    m->n_cells_total = 0;
    m->gall = m->loss_part = m->dwh_part = m->dwh = nullptr;
    m->Xc_all = m->Xn_all = m->tg_all = nullptr;
    m->big = nullptr;
    m->fork = nullptr;
    m->g.resize(m->n_graphs);
    m->off_c.assign(n_graphs + 1, 0); m->off_n.assign(n_graphs + 1, 0);
    m->ux_c.assign(n_graphs, nullptr); m->ux_n.assign(n_graphs, nullptr);
    for (auto& gs : m->g) { gs.stream = nullptr; gs.done = nullptr; gs.X_cell = gs.X_net = nullptr; }
    for (int q = 0; q < n_graphs; ++q) {
        const HeteroDims d = heteroconv_dims(graphs[q]);
        m->off_c[q + 1] = m->off_c[q] + d.Nc;
        m->off_n[q + 1] = m->off_n[q] + d.Nn;
    }
    int rc = DR_OK;
    auto body = [&]() -> int {
        DRC_HIP(hipGetDevice(&m->device));
        DRC_HIP(hipEventCreateWithFlags(&m->fork, hipEventDisableTiming));
        const int L = n_layers, D = m->D;
        std::vector<dr_heteroconv*> ctxs(graphs, graphs + n_graphs);
        if (batched) {
            // ---- stack the sub-graphs' relations into one block-diagonal graph and build its context ----
            const int64_t Nc = m->off_c[n_graphs], Nn = m->off_n[n_graphs];
            for (int r = 0; r < 3; ++r) {
                int64_t nnz = 0;
                for (int q = 0; q < n_graphs; ++q) nnz += heteroconv_relations(graphs[q])[r].nnz;
                DRC_REQUIRE(nnz < (int64_t(1) << 31), "hgnn_create_batched: the stacked graph has 2^31 or more edges in a relation");
                const int64_t rows = (r == 1) ? Nn : Nc, cols = (r == 2) ? Nn : Nc;
                int32_t *rp = nullptr, *ci = nullptr;
                float* v = nullptr;
                DRC_TRY(alloc_t(m, &rp, (size_t)rows + 1));
                DRC_TRY(alloc_t(m, &ci, (size_t)nnz));
                DRC_TRY(alloc_t(m, &v, (size_t)nnz));
                int64_t e0 = 0;
                for (int q = 0; q < n_graphs; ++q) {
                    const dr_csr& A = heteroconv_relations(graphs[q])[r];
                    const int64_t row_off = (r == 1) ? m->off_n[q] : m->off_c[q], col_off = (r == 2) ? m->off_n[q] : m->off_c[q];
                    const int64_t work = A.n_rows > A.nnz ? A.n_rows : A.nnz;
                    unsigned blocks = (unsigned)((work + 255) / 256);
                    blocks = blocks < 1 ? 1 : (blocks > 4096 ? 4096 : blocks);
                    if ((int64_t)blocks * 256 < A.n_rows) blocks = (unsigned)((A.n_rows + 255) / 256);   // one thread per row pointer
                    hipLaunchKernelGGL(concat_csr_kernel, dim3(blocks), dim3(256), 0, nullptr, A.rowptr, A.colidx, A.vals, (int)A.n_rows,
                                       (int)A.nnz, (int)row_off, (int)col_off, (int)e0, q == n_graphs - 1 ? 1 : 0, rp, ci, v);
                    e0 += A.nnz;
                }
                DRC_HIP(hipGetLastError());
                m->big_rel[r] = dr_csr{rows, cols, nnz, rp, ci, v};
            }
            DRC_HIP(hipDeviceSynchronize());
            DRC_TRY(heteroconv_create_widths(&m->big, &m->big_rel[0], &m->big_rel[1], &m->big_rel[2], D, d0.k_near, d0.k_pins,
                                             d0.k_self, d0.k_pinned));
            ctxs.assign(1, m->big);
            DRC_TRY(alloc_t(m, &m->Xc_all, (size_t)Nc * D));
            DRC_TRY(alloc_t(m, &m->Xn_all, (size_t)Nn * D));
            DRC_TRY(alloc_t(m, &m->tg_all, (size_t)Nc));
        }
        const int ns = m->n_graphs;
        DRC_TRY(alloc_t(m, &m->gall, (size_t)ns * m->PL));
        m->n_head_parts = 0;
        // Buffers are sized for the contexts' capacities: a context that a pipeline re-binds to the next sub-graph keeps
        // serving the same model, and every step reads the sizes of the graph that is bound at that moment.
        auto cap_cells = [&](int q) { int64_t c = 0, n = 0; heteroconv_capacity(ctxs[q], &c, &n); return c; };
        auto cap_nets = [&](int q) { int64_t c = 0, n = 0; heteroconv_capacity(ctxs[q], &c, &n); return n; };
        for (int q = 0; q < ns; ++q) m->n_head_parts += head_blocks(cap_cells(q));
        DRC_TRY(alloc_t(m, &m->loss_part, (size_t)m->n_head_parts));
        DRC_TRY(alloc_t(m, &m->dwh_part, (size_t)m->n_head_parts * m->D));
        DRC_TRY(alloc_t(m, &m->dwh, (size_t)m->D));
        int part0 = 0;
        for (int q = 0; q < ns; ++q) {
            GraphState& gs = m->g[q];
            const HeteroDims d = heteroconv_dims(ctxs[q]);
            gs.ctx = ctxs[q]; gs.Nc = d.Nc; gs.Nn = d.Nn;
            const int64_t capc = cap_cells(q), capn = cap_nets(q);
            DRC_REQUIRE(capc >= 1 && capc < (1ll << 31) / D, "hgnn_create: graph %d has room for %lld cells", q, (long long)capc);
            m->n_cells_total += d.Nc;
            DRC_HIP(hipStreamCreateWithFlags(&gs.stream, hipStreamNonBlocking));
            DRC_HIP(hipEventCreateWithFlags(&gs.done, hipEventDisableTiming));
            gs.gvec = m->gall + (size_t)q * m->PL;
            gs.hb = head_blocks(capc);
            gs.loss_part = m->loss_part + (size_t)part0;
            gs.dwh_part = m->dwh_part + (size_t)part0 * D;
            part0 += gs.hb;
            gs.act_c.assign(L, nullptr); gs.act_n.assign(L, nullptr);
            gs.G_c.assign(L + 1, nullptr); gs.G_n.assign(L + 1, nullptr);
            gs.saved.assign(L, dr_heteroconv_saved{});
            const size_t nc = (size_t)capc, nn = (size_t)capn;
            for (int l = 0; l < L; ++l) {
                DRC_TRY(alloc_t(m, &gs.act_c[l], nc * D));
                DRC_TRY(alloc_t(m, &gs.act_n[l], nn * D));
                dr_heteroconv_saved& S = gs.saved[l];
                DRC_TRY(alloc_t(m, &S.vals_cell, nc * d.k_near));
                DRC_TRY(alloc_t(m, &S.idx_cell, nc * d.k_near));
                DRC_TRY(alloc_t(m, &S.vals_net, nn * d.k_pinned));
                DRC_TRY(alloc_t(m, &S.idx_net, nn * d.k_pinned));
                if (d.k_pins != d.k_near) {
                    DRC_TRY(alloc_t(m, &S.vals_cell_pins, nc * d.k_pins));
                    DRC_TRY(alloc_t(m, &S.idx_cell_pins, nc * d.k_pins));
                }
                if (d.k_self != d.k_pinned) {
                    DRC_TRY(alloc_t(m, &S.vals_net_self, nn * d.k_self));
                    DRC_TRY(alloc_t(m, &S.idx_net_self, nn * d.k_self));
                }
                DRC_TRY(alloc_t(m, &S.H_near, nc * D));
                DRC_TRY(alloc_t(m, &S.H_pins, nn * D));
                DRC_TRY(alloc_t(m, &S.H_pinned, nc * D));
                DRC_TRY(alloc_t(m, &S.mask, nc * D));
            }
            for (int l = 0; l <= L; ++l) {
                DRC_TRY(alloc_t(m, &gs.G_c[l], nc * D));
                DRC_TRY(alloc_t(m, &gs.G_n[l], nn * D));
            }
            DRC_TRY(alloc_t(m, &gs.pred, nc));
            DRC_TRY(alloc_t(m, &gs.dpred, nc));
        }
        DRC_HIP(hipDeviceSynchronize());
        if (m->n_graphs > 1) {
            m->pool = new (std::nothrow) EnqueuePool(m->n_graphs < kMaxWorkers ? m->n_graphs : kMaxWorkers, m->device);
            DRC_REQUIRE(m->pool != nullptr, "hgnn_create: out of host memory");
        }
        return DR_OK;
    };
    rc = body();
    if (rc != DR_OK) {
        model_release(m);
        return rc;
    }
    *model = m;
    return DR_OK;
}

// Copies the caller's per-sub-graph blocks behind one another into `dst` unless they already lie that way in
// memory; returns the pointer the step should read.
static int stacked_input(const float* const* parts, int n, const std::vector<int64_t>& off, int width, float* dst,
                         hipStream_t s, const float** out) {
    bool contiguous = true;
    for (int q = 1; q < n && contiguous; ++q) contiguous = parts[q] == parts[0] + (size_t)off[q] * width;
    if (contiguous) { *out = parts[0]; return DR_OK; }
    for (int q0 = 0; q0 < n; q0 += kGatherParts) {
        GatherArgs a;
        a.n = n - q0 < kGatherParts ? n - q0 : kGatherParts;
        for (int i = 0; i < a.n; ++i) {
            a.src[i] = reinterpret_cast<const uint32_t*>(parts[q0 + i]);
            a.start[i] = (unsigned long long)(off[q0 + i] - off[q0]) * width;
        }
        a.start[a.n] = (unsigned long long)(off[q0 + a.n] - off[q0]) * width;
        for (int i = a.n; i < kGatherParts; ++i) { a.src[i] = nullptr; a.start[i + 1] = a.start[a.n]; }
        unsigned long long blocks = (a.start[a.n] + 255) / 256;
        blocks = blocks < 1 ? 1 : (blocks > 8192 ? 8192 : blocks);
        hipLaunchKernelGGL(gather_parts_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a,
                           reinterpret_cast<uint32_t*>(dst + (size_t)off[q0] * width));
    }
    DRC_HIP(hipGetLastError());
    *out = dst;
    return DR_OK;
}

int hgnn_create(dr_hgnn** model, int32_t n_graphs, dr_heteroconv* const* graphs, int32_t n_layers) {
    return create_model(model, n_graphs, graphs, n_layers, false);
}

int hgnn_create_batched(dr_hgnn** model, int32_t n_graphs, dr_heteroconv* const* graphs, int32_t n_layers) {
    return create_model(model, n_graphs, graphs, n_layers, true);
}

int hgnn_train_step(dr_hgnn* m, const float* const* X_cell, const float* const* X_net, const float* const* target,
                    float* theta, float* adam_m, float* adam_v, double lr, double beta1, double beta2, double eps,
                    double weight_decay, int32_t step, float* grad_out, float* loss_out, void* stream) {
    DRC_REQUIRE(m != nullptr, "hgnn_train_step: null model");
    DRC_REQUIRE(X_cell && X_net && target, "hgnn_train_step: null input tables");
    DRC_REQUIRE(theta && adam_m && adam_v && grad_out && loss_out, "hgnn_train_step: null parameter / output vector");
    DRC_REQUIRE(aligned(theta, 16), "hgnn_train_step: theta must be 16-byte aligned");
    DRC_REQUIRE(step >= 1, "hgnn_train_step: step = %d (the first update is step 1)", step);
    DRC_REQUIRE(beta1 >= 0.0 && beta1 < 1.0 && beta2 >= 0.0 && beta2 < 1.0 && eps > 0.0,
                "hgnn_train_step: Adam constants out of range");
    for (int q = 0; q < m->n_user; ++q)
        DRC_REQUIRE(X_cell[q] && X_net[q] && target[q], "hgnn_train_step: null tensor for graph %d", q);
    hipStream_t user = as_stream(stream);
    for (int q = 0; q < m->n_user; ++q) { m->ux_c[q] = X_cell[q]; m->ux_n[q] = X_net[q]; }
    if (!m->batched) {          // the graphs bound to the contexts right now (a pipeline may have re-bound them)
        m->n_cells_total = 0;
        for (auto& gs : m->g) {
            const HeteroDims d = heteroconv_dims(gs.ctx);
            gs.Nc = d.Nc; gs.Nn = d.Nn;
            m->n_cells_total += d.Nc;
        }
    }
    const float *one_c = nullptr, *one_n = nullptr, *one_t = nullptr;      // batched: the stacked inputs
    if (m->batched) {
        DRC_TRY(stacked_input(X_cell, m->n_user, m->off_c, m->D, m->Xc_all, user, &one_c));
        DRC_TRY(stacked_input(X_net, m->n_user, m->off_n, m->D, m->Xn_all, user, &one_n));
        DRC_TRY(stacked_input(target, m->n_user, m->off_c, 1, m->tg_all, user, &one_t));
        X_cell = &one_c; X_net = &one_n; target = &one_t;
    }
    const int L = m->L, D = m->D;
    const float scale = (float)(2.0 / (double)m->n_cells_total);

    DRC_HIP(hipEventRecord(m->fork, user));
    // One sub-graph = one stream = one host thread (of the model's pool): a step of small sub-graphs issues several
    // hundred launches and event operations, and a single host thread cannot enqueue them as fast as the GPU drains them.
    auto enqueue_graph = [&](int q) -> int {
        GraphState& gs = m->g[q];
        hipStream_t s = gs.stream;
        DRC_HIP(hipStreamWaitEvent(s, m->fork, 0));
        gs.X_cell = X_cell[q]; gs.X_net = X_net[q];
        const int n = (int)gs.Nc;
        // ---- forward ----
        const float *xc = X_cell[q], *xn = X_net[q];
        for (int l = 0; l < L; ++l) {
            const dr_heteroconv_weights W = layer_weights(theta, l, D);
            // the ReLU between layers is folded into the kernels that write the layer's outputs
            ForwardOptions fo;
            fo.relu_out = l < L - 1;
            fo.skip_net_output = l == L - 1 && !m->inspect;   // the read-out uses the cells only
            DRC_TRY(heteroconv_forward(gs.ctx, xc, xn, &W, gs.act_c[l], gs.act_n[l], &gs.saved[l], s, fo));
            xc = gs.act_c[l]; xn = gs.act_n[l];
        }
        // ---- read-out, loss, gradient of the last layer's output ----
        const float* w_head = theta + m->PL;
        hipLaunchKernelGGL(head_fwd_kernel, dim3(gs.hb), dim3(256), 0, s, gs.act_c[L - 1], w_head, target[q], n, D,
                           scale, gs.pred, gs.dpred, gs.loss_part);
        hipLaunchKernelGGL(head_bwd_kernel, dim3(gs.hb), dim3(256), 256 * sizeof(float), s, gs.act_c[L - 1], w_head,
                           gs.dpred, n, D, gs.G_c[L], gs.dwh_part);
        DRC_TRY(launch_fill_u32(reinterpret_cast<uint32_t*>(gs.G_n[L]), (size_t)gs.Nn * D, 0u, s));   // nets feed no loss
        DRC_HIP(hipGetLastError());
        // ---- backward ----
        for (int l = L - 1; l >= 0; --l) {
            const dr_heteroconv_weights W = layer_weights(theta, l, D);
            const dr_heteroconv_wgrads dW = layer_wgrads(gs.gvec, l, D);
            // layers above the first sit behind a ReLU: its gate on the input gradient is folded into the kernels
            // that write dX (the saved D-ReLU values are the layer's inputs at every position dX can be non-zero)
            BackwardOptions opt;
            opt.gate_inputs = l >= 1;
            opt.skip_dx = l == 0 && !m->inspect;       // nobody reads the gradient of the input features
            opt.dy_net_zero = l == L - 1;                  // the loss reads the cells only: G_n[L] is the zero fill above
            DRC_TRY(heteroconv_backward(gs.ctx, gs.G_c[l + 1], gs.G_n[l + 1], &W, &gs.saved[l], gs.G_c[l], gs.G_n[l], &dW, s, opt));
        }
        DRC_HIP(hipGetLastError());
        DRC_HIP(hipEventRecord(gs.done, s));
        return DR_OK;
    };
    // Whatever a sub-graph's enqueueing ends with, its `done` event is recorded behind what did get enqueued, and the
    // caller's stream waits for every sub-graph before this call returns -- also when one of them failed, so that no
    // work of this step is still reading theta or the gradient buffers once the caller sees the error.
    const std::function<int(int)> enqueue_and_mark = [&](int q) -> int {
        const int rc = enqueue_graph(q);
        if (rc != DR_OK) (void)hipEventRecord(m->g[q].done, m->g[q].stream);
        return rc;
    };
    int step_rc = DR_OK;
    std::string step_err;
    if (m->n_graphs == 1) {
        step_rc = enqueue_and_mark(0);
        if (step_rc != DR_OK) step_err = dr_last_error();
    } else {
        step_rc = m->pool->run(m->n_graphs, enqueue_and_mark, &step_err);
    }
    if (step_rc != DR_OK) {
        for (int q = 0; q < m->n_graphs; ++q) (void)hipStreamWaitEvent(user, m->g[q].done, 0);
        return fail(step_rc, "%s", step_err.c_str());
    }
    for (int q = 0; q < m->n_graphs; ++q) DRC_HIP(hipStreamWaitEvent(user, m->g[q].done, 0));

    // ---- loss and parameter update, after every sub-graph has delivered its gradient ----
    hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(kWave), 0, user, m->loss_part, m->n_head_parts,
                       (float)(1.0 / (double)m->n_cells_total), loss_out);
    hipLaunchKernelGGL(head_reduce_kernel, dim3((unsigned)D), dim3(256), 0, user, m->dwh_part, m->n_head_parts, D, m->dwh);
    const int64_t P = m->PL + D;
    const float inv_bc1 = (float)(1.0 / (1.0 - std::pow(beta1, (double)step)));
    const float inv_bc2 = (float)(1.0 / (1.0 - std::pow(beta2, (double)step)));
    hipLaunchKernelGGL(adam_kernel, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, user, theta, adam_m, adam_v, grad_out,
                       m->gall, m->dwh, m->n_graphs, m->PL, D, (float)lr, (float)beta1, (float)beta2, (float)(1.0 - beta1),
                       (float)(1.0 - beta2), (float)eps, (float)weight_decay, inv_bc1, inv_bc2);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

int hgnn_get_layer_buffers(const dr_hgnn* m, int32_t graph, int32_t layer, dr_hgnn_layer_buffers* out,
                           const float** pred, const float** dpred) {
    DRC_REQUIRE(m != nullptr && out != nullptr, "hgnn_get_layer_buffers: null argument");
    DRC_REQUIRE(graph >= 0 && graph < m->n_user, "hgnn_get_layer_buffers: graph %d out of range", graph);
    DRC_REQUIRE(layer >= 0 && layer < m->L, "hgnn_get_layer_buffers: layer %d out of range", layer);
    // a batched model holds one stacked state: sub-graph q's rows start at off_c[q] / off_n[q] in every buffer
    const GraphState& gs = m->g[m->batched ? 0 : graph];
    const size_t oc = m->batched ? (size_t)m->off_c[graph] : 0, on = m->batched ? (size_t)m->off_n[graph] : 0;
    const size_t D = (size_t)m->D;
    const HeteroDims d = heteroconv_dims(gs.ctx);
    out->X_cell = layer == 0 ? m->ux_c[graph] : gs.act_c[layer - 1] + oc * D;
    out->X_net = layer == 0 ? m->ux_n[graph] : gs.act_n[layer - 1] + on * D;
    out->Y_cell = gs.act_c[layer] + oc * D;
    const bool has_net_out = layer < m->L - 1 || m->inspect;
    out->Y_net = has_net_out ? gs.act_n[layer] + on * D : nullptr;
    const dr_heteroconv_saved& S = gs.saved[layer];
    dr_heteroconv_saved& o = out->saved;
    o = dr_heteroconv_saved{};
    o.vals_cell = S.vals_cell + oc * d.k_near;   o.idx_cell = S.idx_cell + oc * d.k_near;
    o.vals_net = S.vals_net + on * d.k_pinned;   o.idx_net = S.idx_net + on * d.k_pinned;
    o.H_near = S.H_near + oc * D; o.H_pins = has_net_out ? S.H_pins + on * D : nullptr; o.H_pinned = S.H_pinned + oc * D;
    o.mask = S.mask + oc * D;
    if (S.vals_cell_pins) { o.vals_cell_pins = S.vals_cell_pins + oc * d.k_pins; o.idx_cell_pins = S.idx_cell_pins + oc * d.k_pins; }
    if (S.vals_net_self) { o.vals_net_self = S.vals_net_self + on * d.k_self; o.idx_net_self = S.idx_net_self + on * d.k_self; }
    out->dY_cell = gs.G_c[layer + 1] + oc * D;
    out->dY_net = gs.G_n[layer + 1] + on * D;
    const bool has_dx = layer > 0 || m->inspect;
    out->dX_cell = has_dx ? gs.G_c[layer] + oc * D : nullptr;
    out->dX_net = has_dx ? gs.G_n[layer] + on * D : nullptr;
    out->dW = layer_wgrads(gs.gvec, layer, m->D);       // batched: of the whole batch, whichever sub-graph is asked for
    if (pred) *pred = gs.pred + oc;
    if (dpred) *dpred = gs.dpred + oc;
    return DR_OK;
}

int hgnn_set_inspection(dr_hgnn* m, int enable) {
    DRC_REQUIRE(m != nullptr, "hgnn_set_inspection: null model");
    m->inspect = enable != 0;
    return DR_OK;
}

int hgnn_destroy(dr_hgnn* m) {
    if (!m) return DR_OK;
    (void)hipDeviceSynchronize();
    model_release(m);
    return DR_OK;
}

}  // extern "C"
