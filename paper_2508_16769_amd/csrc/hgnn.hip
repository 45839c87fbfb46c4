// Multi-layer training step (paper Section 4.1): L stacked HeteroConv layers with ReLU between them, a
// per-cell read-out pred = X_cell^(L) . w_head, mean-squared error over all cells of the batch, Adam with
// the L2 form of weight decay.  The sub-graphs of a batch are independent (Section 3.4): each runs its
// whole forward and backward on its own stream (the relation streams of its layer context fork below
// that), and the streams are joined only before the parameter update.
//
// What is new here next to the layer is element-wise or a small reduction:
//   relu_inplace / relu_bwd_inplace   activation and its gate, in place on the layer outputs / gradients
//   head_fwd_kernel                    one wavefront per cell: dot product, residual, loss partials
//   head_bwd_kernel                    dY = dpred (x) w_head, per-workgroup partials of dw_head = Y^T dpred
//   loss_reduce_kernel, adam_kernel    fixed-order sums over sub-graphs and partials, then the update
// Every sum has a fixed order, so a step is reproducible bit for bit.
#include "dr_internal.h"

#include <cmath>
#include <new>
#include <string>
#include <thread>
#include <vector>

namespace drc {

constexpr int kHeadBlocks = 64;   // workgroups (partials) per sub-graph in the read-out kernels
constexpr int kMaxWorkers = 8;    // host threads that enqueue sub-graphs side by side

__global__ __launch_bounds__(256) void relu_inplace(float4* __restrict__ y, size_t n4) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
        float4 v = y[i];
        v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f);
        y[i] = v;
    }
}

// dx = act > 0 ? dx : 0   (act is the ReLU output, so act > 0 exactly where its input was > 0)
__global__ __launch_bounds__(256) void relu_bwd_inplace(float4* __restrict__ dx, const float4* __restrict__ act, size_t n4) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
        float4 g = dx[i];
        const float4 a = act[i];
        g.x = a.x > 0.f ? g.x : 0.f; g.y = a.y > 0.f ? g.y : 0.f; g.z = a.z > 0.f ? g.z : 0.f; g.w = a.w > 0.f ? g.w : 0.f;
        dx[i] = g;
    }
}

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

// g = sum over sub-graphs (fixed order) of the gradient pieces; Adam with L2 weight decay, bias-corrected
__global__ __launch_bounds__(256) void adam_kernel(float* __restrict__ theta, float* __restrict__ m, float* __restrict__ v,
                                                   float* __restrict__ grad_out, const float* __restrict__ gall,
                                                   const float* __restrict__ dwh_part, int n_graphs, int64_t PL, int D,
                                                   float lr, float beta1, float beta2, float omb1, float omb2,
                                                   float eps, float wd, float inv_bc1, float inv_bc2) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= PL + D) return;
    float g = 0.f;
    if (e < PL) {
        for (int q = 0; q < n_graphs; ++q) g += gall[(size_t)q * PL + e];
    } else {
        const int c = (int)(e - PL);
        for (int q = 0; q < n_graphs * kHeadBlocks; ++q) g += dwh_part[(size_t)q * D + c];
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

struct GraphState {
    dr_heteroconv* ctx;
    int64_t Nc, Nn;
    std::vector<float*> act_c, act_n;          // [L] layer outputs
    std::vector<dr_heteroconv_saved> saved;    // [L]
    std::vector<float*> G_c, G_n;              // [L+1] gradients: G[l] = dX of layer l = (after the gate) dY of layer l-1
    float* gvec;                               // this sub-graph's layer-weight gradients, theta layout (slice of gall)
    float *pred, *dpred;
    float *loss_part, *dwh_part;               // slices of the model's partial arrays
    hipStream_t stream;
    hipEvent_t done;
    const float *X_cell, *X_net;               // caller's inputs of the last step (for inspection)
};

}  // namespace drc

struct dr_hgnn {
    int n_graphs, L, D;
    int64_t PL;                                // layer parameters: L*5*D*D
    int64_t n_cells_total;
    std::vector<drc::GraphState> g;
    std::vector<void*> owned;
    float *gall, *loss_part, *dwh_part;
    hipEvent_t fork;
    int device;
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
    for (void* p : m->owned) (void)hipFree(p);
    for (auto& gs : m->g) {
        if (gs.stream) (void)hipStreamDestroy(gs.stream);
        if (gs.done) (void)hipEventDestroy(gs.done);
    }
    if (m->fork) (void)hipEventDestroy(m->fork);
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

unsigned ew_blocks(size_t n4) {
    size_t b = (n4 + 255) / 256;
    return (unsigned)(b > 4096 ? 4096 : (b < 1 ? 1 : b));
}

}  // namespace

extern "C" {

int64_t hgnn_num_params(int32_t n_layers, int32_t D) {
    if (n_layers < 1 || D < 1) return 0;
    return (int64_t)n_layers * 5 * D * D + D;
}

int hgnn_create(dr_hgnn** model, int32_t n_graphs, dr_heteroconv* const* graphs, int32_t n_layers) {
    DRC_REQUIRE(model != nullptr, "hgnn_create: null model");
    *model = nullptr;
    DRC_REQUIRE(n_graphs >= 1 && n_graphs <= 1024, "hgnn_create: n_graphs = %d out of range [1, 1024]", n_graphs);
    DRC_REQUIRE(n_layers >= 1 && n_layers <= 16, "hgnn_create: n_layers = %d out of range [1, 16]", n_layers);
    DRC_REQUIRE(graphs != nullptr, "hgnn_create: null graphs");
    for (int q = 0; q < n_graphs; ++q) DRC_REQUIRE(graphs[q] != nullptr, "hgnn_create: graph %d is null", q);
    for (int q = 0; q < n_graphs; ++q)
        for (int r = 0; r < q; ++r)
            DRC_REQUIRE(graphs[q] != graphs[r], "hgnn_create: graphs %d and %d share one context (its scratch is per step)", r, q);
    const HeteroDims d0 = heteroconv_dims(graphs[0]);
    for (int q = 1; q < n_graphs; ++q) {   // the parameters are shared, so the width is; each sub-graph keeps its own K
        const HeteroDims d = heteroconv_dims(graphs[q]);
        DRC_REQUIRE(d.D == d0.D, "hgnn_create: graph %d has D = %d, graph 0 has %d", q, d.D, d0.D);
    }
    dr_hgnn* m = new (std::nothrow) dr_hgnn();
    if (!m) return fail(DR_ERR_HIP, "hgnn_create: out of host memory");
    m->n_graphs = n_graphs; m->L = n_layers; m->D = d0.D;
    m->PL = (int64_t)n_layers * 5 * d0.D * d0.D;
    m->n_cells_total = 0;
    m->gall = m->loss_part = m->dwh_part = nullptr;
    m->fork = nullptr;
    m->g.resize(n_graphs);
    for (auto& gs : m->g) { gs.stream = nullptr; gs.done = nullptr; gs.X_cell = gs.X_net = nullptr; }
    int rc = DR_OK;
    auto body = [&]() -> int {
        DRC_HIP(hipGetDevice(&m->device));
        DRC_HIP(hipEventCreateWithFlags(&m->fork, hipEventDisableTiming));
        DRC_TRY(alloc_t(m, &m->gall, (size_t)n_graphs * m->PL));
        DRC_TRY(alloc_t(m, &m->loss_part, (size_t)n_graphs * kHeadBlocks));
        DRC_TRY(alloc_t(m, &m->dwh_part, (size_t)n_graphs * kHeadBlocks * m->D));
        const int L = n_layers, D = m->D;
        for (int q = 0; q < n_graphs; ++q) {
            GraphState& gs = m->g[q];
            const HeteroDims d = heteroconv_dims(graphs[q]);
            gs.ctx = graphs[q]; gs.Nc = d.Nc; gs.Nn = d.Nn;
            DRC_REQUIRE(d.Nc >= 1 && d.Nc < (1ll << 31) / D, "hgnn_create: graph %d has %lld cells", q, (long long)d.Nc);
            m->n_cells_total += d.Nc;
            DRC_HIP(hipStreamCreateWithFlags(&gs.stream, hipStreamNonBlocking));
            DRC_HIP(hipEventCreateWithFlags(&gs.done, hipEventDisableTiming));
            gs.gvec = m->gall + (size_t)q * m->PL;
            gs.loss_part = m->loss_part + (size_t)q * kHeadBlocks;
            gs.dwh_part = m->dwh_part + (size_t)q * kHeadBlocks * D;
            gs.act_c.assign(L, nullptr); gs.act_n.assign(L, nullptr);
            gs.G_c.assign(L + 1, nullptr); gs.G_n.assign(L + 1, nullptr);
            gs.saved.assign(L, dr_heteroconv_saved{});
            const size_t nc = (size_t)d.Nc, nn = (size_t)d.Nn;
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
    for (int q = 0; q < m->n_graphs; ++q)
        DRC_REQUIRE(X_cell[q] && X_net[q] && target[q], "hgnn_train_step: null tensor for graph %d", q);
    hipStream_t user = as_stream(stream);
    const int L = m->L, D = m->D;
    const float scale = (float)(2.0 / (double)m->n_cells_total);

    DRC_HIP(hipEventRecord(m->fork, user));
    // One sub-graph = one stream = one host thread: a step of small sub-graphs issues several hundred launches
    // and event operations, and a single host thread cannot enqueue them as fast as the GPU drains them.
    auto enqueue_graph = [&](int q) -> int {
        GraphState& gs = m->g[q];
        hipStream_t s = gs.stream;
        DRC_HIP(hipStreamWaitEvent(s, m->fork, 0));
        gs.X_cell = X_cell[q]; gs.X_net = X_net[q];
        const int n = (int)gs.Nc;
        const size_t c4 = (size_t)gs.Nc * D / 4, n4 = (size_t)gs.Nn * D / 4;
        // ---- forward ----
        const float *xc = X_cell[q], *xn = X_net[q];
        for (int l = 0; l < L; ++l) {
            const dr_heteroconv_weights W = layer_weights(theta, l, D);
            DRC_TRY(heteroconv_fwd(gs.ctx, xc, xn, &W, gs.act_c[l], gs.act_n[l], &gs.saved[l], s));
            if (l < L - 1) {
                hipLaunchKernelGGL(relu_inplace, dim3(ew_blocks(c4)), dim3(256), 0, s, reinterpret_cast<float4*>(gs.act_c[l]), c4);
                hipLaunchKernelGGL(relu_inplace, dim3(ew_blocks(n4)), dim3(256), 0, s, reinterpret_cast<float4*>(gs.act_n[l]), n4);
            }
            xc = gs.act_c[l]; xn = gs.act_n[l];
        }
        // ---- read-out, loss, gradient of the last layer's output ----
        const float* w_head = theta + m->PL;
        hipLaunchKernelGGL(head_fwd_kernel, dim3(kHeadBlocks), dim3(256), 0, s, gs.act_c[L - 1], w_head, target[q], n, D,
                           scale, gs.pred, gs.dpred, gs.loss_part);
        hipLaunchKernelGGL(head_bwd_kernel, dim3(kHeadBlocks), dim3(256), 256 * sizeof(float), s, gs.act_c[L - 1], w_head,
                           gs.dpred, n, D, gs.G_c[L], gs.dwh_part);
        DRC_TRY(launch_fill_u32(reinterpret_cast<uint32_t*>(gs.G_n[L]), (size_t)gs.Nn * D, 0u, s));   // nets feed no loss
        DRC_HIP(hipGetLastError());
        // ---- backward ----
        for (int l = L - 1; l >= 0; --l) {
            const dr_heteroconv_weights W = layer_weights(theta, l, D);
            const dr_heteroconv_wgrads dW = layer_wgrads(gs.gvec, l, D);
            DRC_TRY(heteroconv_bwd(gs.ctx, gs.G_c[l + 1], gs.G_n[l + 1], &W, &gs.saved[l], gs.G_c[l], gs.G_n[l], &dW, s));
            if (l >= 1) {   // gate by the ReLU in front of layer l: its output is the input of layer l
                hipLaunchKernelGGL(relu_bwd_inplace, dim3(ew_blocks(c4)), dim3(256), 0, s, reinterpret_cast<float4*>(gs.G_c[l]),
                                   reinterpret_cast<const float4*>(gs.act_c[l - 1]), c4);
                hipLaunchKernelGGL(relu_bwd_inplace, dim3(ew_blocks(n4)), dim3(256), 0, s, reinterpret_cast<float4*>(gs.G_n[l]),
                                   reinterpret_cast<const float4*>(gs.act_n[l - 1]), n4);
            }
        }
        DRC_HIP(hipGetLastError());
        DRC_HIP(hipEventRecord(gs.done, s));
        return DR_OK;
    };
    if (m->n_graphs == 1) {
        DRC_TRY(enqueue_graph(0));
    } else {
        const int n_workers = m->n_graphs < kMaxWorkers ? m->n_graphs : kMaxWorkers;
        std::vector<int> rcs(n_workers, DR_OK);
        std::vector<std::string> errs(n_workers);
        std::vector<std::thread> workers;
        workers.reserve(n_workers);
        for (int w = 0; w < n_workers; ++w)
            workers.emplace_back([&, w]() {
                if (hipSetDevice(m->device) != hipSuccess) { rcs[w] = DR_ERR_HIP; errs[w] = "hipSetDevice failed in a worker thread"; return; }
                for (int q = w; q < m->n_graphs && rcs[w] == DR_OK; q += n_workers) rcs[w] = enqueue_graph(q);
                if (rcs[w] != DR_OK) errs[w] = dr_last_error();      // the error text is per thread: hand it over
            });
        for (auto& t : workers) t.join();
        for (int w = 0; w < n_workers; ++w)
            if (rcs[w] != DR_OK) return fail(rcs[w], "%s", errs[w].c_str());
    }
    for (int q = 0; q < m->n_graphs; ++q) DRC_HIP(hipStreamWaitEvent(user, m->g[q].done, 0));

    // ---- loss and parameter update, after every sub-graph has delivered its gradient ----
    hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(kWave), 0, user, m->loss_part, m->n_graphs * kHeadBlocks,
                       (float)(1.0 / (double)m->n_cells_total), loss_out);
    const int64_t P = m->PL + D;
    const float inv_bc1 = (float)(1.0 / (1.0 - std::pow(beta1, (double)step)));
    const float inv_bc2 = (float)(1.0 / (1.0 - std::pow(beta2, (double)step)));
    hipLaunchKernelGGL(adam_kernel, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, user, theta, adam_m, adam_v, grad_out,
                       m->gall, m->dwh_part, m->n_graphs, m->PL, D, (float)lr, (float)beta1, (float)beta2, (float)(1.0 - beta1),
                       (float)(1.0 - beta2), (float)eps, (float)weight_decay, inv_bc1, inv_bc2);
    DRC_HIP(hipGetLastError());
    return DR_OK;
}

int hgnn_get_layer_buffers(const dr_hgnn* m, int32_t graph, int32_t layer, dr_hgnn_layer_buffers* out,
                           const float** pred, const float** dpred) {
    DRC_REQUIRE(m != nullptr && out != nullptr, "hgnn_get_layer_buffers: null argument");
    DRC_REQUIRE(graph >= 0 && graph < m->n_graphs, "hgnn_get_layer_buffers: graph %d out of range", graph);
    DRC_REQUIRE(layer >= 0 && layer < m->L, "hgnn_get_layer_buffers: layer %d out of range", layer);
    const GraphState& gs = m->g[graph];
    out->X_cell = layer == 0 ? gs.X_cell : gs.act_c[layer - 1];
    out->X_net = layer == 0 ? gs.X_net : gs.act_n[layer - 1];
    out->Y_cell = gs.act_c[layer];
    out->Y_net = gs.act_n[layer];
    out->saved = gs.saved[layer];
    out->dY_cell = gs.G_c[layer + 1];
    out->dY_net = gs.G_n[layer + 1];
    out->dX_cell = gs.G_c[layer];
    out->dX_net = gs.G_n[layer];
    out->dW = layer_wgrads(gs.gvec, layer, m->D);
    if (pred) *pred = gs.pred;
    if (dpred) *dpred = gs.dpred;
    return DR_OK;
}

int hgnn_destroy(dr_hgnn* m) {
    if (!m) return DR_OK;
    (void)hipDeviceSynchronize();
    model_release(m);
    return DR_OK;
}

}  // extern "C"
