// HeteroConv layer: per-graph context and the forward / backward schedules.  The three relation
// pipelines (near, pins, pinned) run on three HIP streams of the one GPU and are joined by events only
// where the data flow demands it (paper Section 3.4: independent sub-graph updates launched together,
// merged at the cell node type).  The host never waits inside fwd / bwd.
#include "dr_internal.h"

#include <new>
#include <vector>

namespace {
// kernel ids for the optional per-kernel timing (heteroconv_profile / heteroconv_kernel_times)
enum KernelId {
    kTopkCell, kTopkNet, kFwdNear, kFwdPins, kFwdPinned, kProjNear, kProjPins, kProjPinnedMerge,
    kDhNear, kBwdNear, kWgNear, kDhPins, kBwdPins, kSelfNearSample,
    kWgPins, kDhPinned, kBwdPinned, kSelfPinsSample, kWgPinned, kNumKernels
};
const char* const kKernelNames[kNumKernels] = {
    "dr_topk.cell", "dr_topk.net", "dr_spmm_fwd.near", "dr_spmm_fwd.pins", "dr_spmm_fwd.pinned",
    "proj.near", "proj.pins", "proj.pinned+merge",
    "dproj.near", "dr_spmm_bwd.near", "wgrad.near", "dproj.pins", "dr_spmm_bwd.pins",
    "dself.near+dX", "wgrad.pins", "dproj.pinned",
    "dr_spmm_bwd.pinned", "dself.pins+dX", "wgrad.pinned"};
struct TimedLaunch { int id; hipEvent_t start, stop; bool start_shared; };   // start_shared: start is the previous launch's stop
}  // namespace

struct dr_heteroconv {
    int64_t Nc, Nn;
    int D;
    // D-ReLU widths: k_near (cells, source and self term of near), k_pins (cells, source of pins), k_self (nets,
    // self term of pins), k_pinned (nets, source of pinned).  Equal widths on one node type share one CBSR.
    int k_near, k_pins, k_self, k_pinned;
    dr_csr A[3];        // near, pins, pinned (borrowed)
    dr_csr At[3];       // transposes (owned)
    // what the owned buffers were sized for; a context can be re-bound to any graph within these bounds
    int64_t cap_Nc, cap_Nn, cap_E[3];
    int32_t* t_rp[3];   // buffers behind At[]
    int32_t* t_ci[3];
    float* t_v[3];
    void* t_ws[3];      // transpose workspaces (kept only by re-bindable contexts)
    size_t t_wsb[3];
    void* owned[32];
    int n_owned;
    hipStream_t st[3];  // near, pins, pinned
    hipEvent_t ev_fork, ev_topk_cell, ev_topk_net, ev_near, ev_pins, ev_pinned, ev_gnear, ev_gpins;
    // backward scratch
    float* dH[3];       // [Nc,D], [Nn,D], [Nc,D]
    float* dXs_cell;    // [Nc,k_near]  compact gradient at the near selection (both cell pieces when k_pins == k_near)
    float* dXs_cell_b;  // [Nc,k_pins]  pins piece at its own selection (only when k_pins != k_near)
    float* dXs_net;     // [Nn,k_pinned]
    float* wg_scratch[3];
    int device;
    int overlap;        // DR_OVERLAP_*: whether the relation pipelines run on separate streams
    dr_spmm_plan* near_plan;   // transposed `near` with its dH rows staged in LDS tile by tile (heteroconv_set_cell_order), or null
    // optional per-kernel timing
    bool profile;
    std::vector<TimedLaunch>* timed;      // launches recorded since the last heteroconv_kernel_times
    std::vector<hipEvent_t>* event_pool;  // idle timing events
    hipEvent_t chain_stop;                // stop event of the previous timed launch of this call, when it can serve
    hipStream_t chain_stream;             //   as the start of the next one (same stream, nothing but launches between)
    bool chain_ok;                        // all relations on one stream: consecutive launches run back to back
};

using namespace drc;

// Staging the gathered rows of a tile pays from about two edges per staged row on (measured on the 1.2 M-cell `near`
// relation: 0.64 ms at 2.1, 0.42 ms at 4.7, against 0.67 ms for the plain gather).
static constexpr double kMinStagingReuse = 2.0;

HeteroDims drc::heteroconv_dims(const dr_heteroconv* c) {
    return HeteroDims{c->Nc, c->Nn, c->D, c->k_near, c->k_pins, c->k_self, c->k_pinned};
}

namespace {

int dev_alloc(dr_heteroconv* c, void** p, size_t bytes) {
    *p = nullptr;
    if (bytes == 0) bytes = 256;
    DRC_HIP(hipMalloc(p, bytes));
    c->owned[c->n_owned++] = *p;
    return DR_OK;
}

void release(dr_heteroconv* c) {
    if (!c) return;
    spmm_plan_destroy(c->near_plan);
    for (int i = 0; i < c->n_owned; ++i) (void)hipFree(c->owned[i]);
    for (int i = 0; i < 3; ++i)
        if (c->st[i]) (void)hipStreamDestroy(c->st[i]);
    hipEvent_t* evs[] = {&c->ev_fork, &c->ev_topk_cell, &c->ev_topk_net, &c->ev_near,
                         &c->ev_pins, &c->ev_pinned, &c->ev_gnear, &c->ev_gpins};
    for (hipEvent_t* e : evs)
        if (*e) (void)hipEventDestroy(*e);
    if (c->timed) {
        for (TimedLaunch& t : *c->timed) { if (!t.start_shared) (void)hipEventDestroy(t.start); (void)hipEventDestroy(t.stop); }
        delete c->timed;
    }
    if (c->event_pool) {
        for (hipEvent_t e : *c->event_pool) (void)hipEventDestroy(e);
        delete c->event_pool;
    }
    delete c;
}

// Brackets one launch with timing events on its own stream when profiling is on.  With all relations on one
// stream the launches of a call run back to back, so the stop event of one launch also serves as the start of
// the next: one event record per launch instead of two (each record is a packet the GPU has to process).
struct ScopedTiming {
    dr_heteroconv* c; hipStream_t s; TimedLaunch t; bool on;
    hipEvent_t take() {
        hipEvent_t e = nullptr;
        if (!c->event_pool->empty()) { e = c->event_pool->back(); c->event_pool->pop_back(); }
        else if (hipEventCreate(&e) != hipSuccess) e = nullptr;
        return e;
    }
    ScopedTiming(dr_heteroconv* c_, int id, hipStream_t s_) : c(c_), s(s_), t{id, nullptr, nullptr, false}, on(false) {
        if (!c->profile) return;
        if (c->chain_ok && c->chain_stop && c->chain_stream == s) {
            t.start = c->chain_stop;
            t.start_shared = true;
            t.stop = take();
            on = t.stop != nullptr;
        } else {
            t.start = take();
            t.stop = take();
            if (t.start && t.stop && hipEventRecord(t.start, s) == hipSuccess) on = true;
        }
    }
    ~ScopedTiming() {
        if (!on) return;
        (void)hipEventRecord(t.stop, s);
        c->timed->push_back(t);
        c->chain_stop = t.stop;
        c->chain_stream = s;
    }
};

}  // namespace

const dr_csr* drc::heteroconv_relations(const dr_heteroconv* c) { return c->A; }

void drc::heteroconv_capacity(const dr_heteroconv* c, int64_t* cells, int64_t* nets) { *cells = c->cap_Nc; *nets = c->cap_Nn; }

static int check_widths(int32_t D, int32_t k_near, int32_t k_pins, int32_t k_self, int32_t k_pinned) {
    DRC_REQUIRE(k_near >= 1 && k_pins >= 1 && k_self >= 1 && k_pinned >= 1, "heteroconv_create: k must be >= 1");
    DRC_REQUIRE(k_near <= D && k_pins <= D && k_self <= D && k_pinned <= D, "heteroconv_create: k exceeds D");
    if (!(D == 32 || D == 64 || D == 96 || D == 128))
        return fail(DR_ERR_UNSUPPORTED, "heteroconv_create: D = %d not in {32,64,96,128}", D);
    return DR_OK;
}

int drc::heteroconv_create_capacity(dr_heteroconv** ctx, int64_t Nc, int64_t Nn, const int64_t E[3], int32_t D, int32_t k_near,
                                    int32_t k_pins, int32_t k_self, int32_t k_pinned, bool keep_workspace) {
    DRC_REQUIRE(ctx != nullptr, "heteroconv_create: null ctx");
    *ctx = nullptr;
    DRC_TRY(check_widths(D, k_near, k_pins, k_self, k_pinned));
    DRC_REQUIRE(Nc >= 0 && Nn >= 0 && E[0] >= 0 && E[1] >= 0 && E[2] >= 0, "heteroconv_create: negative size");
    DRC_REQUIRE(E[0] < (int64_t(1) << 31) && E[1] < (int64_t(1) << 31) && E[2] < (int64_t(1) << 31), "heteroconv_create: nnz >= 2^31");
    DRC_REQUIRE(Nc * (int64_t)D < (int64_t(1) << 31) * 2 && Nn * (int64_t)D < (int64_t(1) << 31) * 2,
                "heteroconv_create: n*D too large");

    dr_heteroconv* c = new (std::nothrow) dr_heteroconv();
    DRC_REQUIRE(c != nullptr, "heteroconv_create: out of host memory");
    c->Nc = Nc; c->Nn = Nn; c->D = D;
    c->cap_Nc = Nc; c->cap_Nn = Nn;
    for (int i = 0; i < 3; ++i) c->cap_E[i] = E[i];
    c->k_near = k_near; c->k_pins = k_pins; c->k_self = k_self; c->k_pinned = k_pinned;
    c->timed = new (std::nothrow) std::vector<TimedLaunch>();
    c->event_pool = new (std::nothrow) std::vector<hipEvent_t>();

    int rc = DR_OK;
    auto bail = [&](int code) { release(c); return code; };
    if (hipGetDevice(&c->device) != hipSuccess) return bail(hip_fail(hipGetLastError(), "hipGetDevice"));
    for (int i = 0; i < 3; ++i)
        if (hipStreamCreateWithFlags(&c->st[i], hipStreamNonBlocking) != hipSuccess)
            return bail(hip_fail(hipGetLastError(), "hipStreamCreateWithFlags"));
    hipEvent_t* evs[] = {&c->ev_fork, &c->ev_topk_cell, &c->ev_topk_net, &c->ev_near,
                         &c->ev_pins, &c->ev_pinned, &c->ev_gnear, &c->ev_gpins};
    for (hipEvent_t* e : evs)
        if (hipEventCreateWithFlags(e, hipEventDisableTiming) != hipSuccess)
            return bail(hip_fail(hipGetLastError(), "hipEventCreateWithFlags"));

    // buffers of the transposed adjacencies: A^T of relation i has as many rows as A has columns
    const int64_t t_rows[3] = {Nc, Nc, Nn}, a_rows[3] = {Nc, Nn, Nc};
    for (int i = 0; i < 3; ++i) {
        if ((rc = dev_alloc(c, (void**)&c->t_rp[i], 4 * (size_t)(t_rows[i] + 1)))) return bail(rc);
        if ((rc = dev_alloc(c, (void**)&c->t_ci[i], 4 * (size_t)E[i]))) return bail(rc);
        if ((rc = dev_alloc(c, (void**)&c->t_v[i], 4 * (size_t)E[i]))) return bail(rc);
        c->t_wsb[i] = dr_csr_transpose_workspace_bytes(a_rows[i], t_rows[i], E[i]);
        if (keep_workspace && (rc = dev_alloc(c, &c->t_ws[i], c->t_wsb[i]))) return bail(rc);
    }
    const int64_t drows[3] = {Nc, Nn, Nc};
    for (int i = 0; i < 3; ++i) {
        if ((rc = dev_alloc(c, (void**)&c->dH[i], 4 * (size_t)drows[i] * D))) return bail(rc);
        if ((rc = dev_alloc(c, (void**)&c->wg_scratch[i], wgrad_scratch_bytes(Nc > Nn ? Nc : Nn, D)))) return bail(rc);
    }
    if ((rc = dev_alloc(c, (void**)&c->dXs_cell, 4 * (size_t)Nc * k_near))) return bail(rc);
    if (k_pins != k_near && (rc = dev_alloc(c, (void**)&c->dXs_cell_b, 4 * (size_t)Nc * k_pins))) return bail(rc);
    if ((rc = dev_alloc(c, (void**)&c->dXs_net, 4 * (size_t)Nn * k_pinned))) return bail(rc);
    *ctx = c;
    return DR_OK;
}

// Binds three relations (device CSRs within the context's capacity) and enqueues their transposition on `s`.
// Nothing here waits for the device; work enqueued on the context after `s` has passed this point sees the new graph.
int drc::heteroconv_bind(dr_heteroconv* c, const dr_csr* near, const dr_csr* pins, const dr_csr* pinned, hipStream_t s) {
    if (int rc = check_csr(near, "heteroconv_bind: near", true)) return rc;
    if (int rc = check_csr(pins, "heteroconv_bind: pins", true)) return rc;
    if (int rc = check_csr(pinned, "heteroconv_bind: pinned", true)) return rc;
    DRC_REQUIRE(near->n_rows == near->n_cols, "heteroconv_bind: near must be square (cell x cell)");
    const int64_t Nc = near->n_rows, Nn = pins->n_rows;
    DRC_REQUIRE(pins->n_cols == Nc, "heteroconv_bind: pins must be Nn x Nc");
    DRC_REQUIRE(pinned->n_rows == Nc && pinned->n_cols == Nn, "heteroconv_bind: pinned must be Nc x Nn");
    DRC_REQUIRE(Nc <= c->cap_Nc && Nn <= c->cap_Nn && near->nnz <= c->cap_E[0] && pins->nnz <= c->cap_E[1] &&
                    pinned->nnz <= c->cap_E[2],
                "heteroconv_bind: graph (%lld cells, %lld nets, %lld / %lld / %lld edges) exceeds the context's capacity",
                (long long)Nc, (long long)Nn, (long long)near->nnz, (long long)pins->nnz, (long long)pinned->nnz);
    c->Nc = Nc; c->Nn = Nn;
    c->A[0] = *near; c->A[1] = *pins; c->A[2] = *pinned;
    if (c->near_plan) {      // made for the graph bound before
        DRC_HIP(hipDeviceSynchronize());
        spmm_plan_destroy(c->near_plan);
        c->near_plan = nullptr;
    }
    for (int i = 0; i < 3; ++i) {
        const dr_csr& A = c->A[i];
        DRC_REQUIRE(c->t_ws[i] != nullptr, "heteroconv_bind: context without transpose workspace");
        DRC_TRY(dr_csr_transpose(&A, c->t_rp[i], c->t_ci[i], c->t_v[i], c->t_ws[i], c->t_wsb[i], s));
        c->At[i] = dr_csr{A.n_cols, A.n_rows, A.nnz, c->t_rp[i], c->t_ci[i], c->t_v[i]};
    }
    return DR_OK;
}

int drc::heteroconv_create_widths(dr_heteroconv** ctx, const dr_csr* near, const dr_csr* pins, const dr_csr* pinned, int32_t D,
                                  int32_t k_near, int32_t k_pins, int32_t k_self, int32_t k_pinned) {
    DRC_REQUIRE(ctx != nullptr, "heteroconv_create: null ctx");
    *ctx = nullptr;
    if (int rc = check_csr(near, "heteroconv_create: near", true)) return rc;
    if (int rc = check_csr(pins, "heteroconv_create: pins", true)) return rc;
    if (int rc = check_csr(pinned, "heteroconv_create: pinned", true)) return rc;
    DRC_REQUIRE(near->n_rows == near->n_cols, "heteroconv_create: near must be square (cell x cell)");
    const int64_t Nc = near->n_rows, Nn = pins->n_rows;
    DRC_REQUIRE(pins->n_cols == Nc, "heteroconv_create: pins must be Nn x Nc");
    DRC_REQUIRE(pinned->n_rows == Nc && pinned->n_cols == Nn, "heteroconv_create: pinned must be Nc x Nn");
    DRC_TRY(check_widths(D, k_near, k_pins, k_self, k_pinned));
    // the caller may still be producing the CSR arrays on another stream
    DRC_HIP(hipDeviceSynchronize());
    const int64_t E[3] = {near->nnz, pins->nnz, pinned->nnz};
    dr_heteroconv* c = nullptr;
    DRC_TRY(heteroconv_create_capacity(&c, Nc, Nn, E, D, k_near, k_pins, k_self, k_pinned, false));
    // one-off transposition: the workspaces are released again
    int rc = DR_OK;
    for (int i = 0; i < 3 && rc == DR_OK; ++i)
        if (hipMalloc(&c->t_ws[i], c->t_wsb[i] ? c->t_wsb[i] : 256) != hipSuccess) rc = hip_fail(hipGetLastError(), "hipMalloc(transpose workspace)");
    if (rc == DR_OK) rc = heteroconv_bind(c, near, pins, pinned, c->st[0]);
    const hipError_t e = hipDeviceSynchronize();
    for (int i = 0; i < 3; ++i) {
        if (c->t_ws[i]) (void)hipFree(c->t_ws[i]);
        c->t_ws[i] = nullptr;
    }
    if (rc == DR_OK && e != hipSuccess) rc = hip_fail(e, "hipDeviceSynchronize(transpose)");
    if (rc != DR_OK) { release(c); return rc; }
    *ctx = c;
    return DR_OK;
}

extern "C" {

int heteroconv_create(dr_heteroconv** ctx, const dr_csr* near, const dr_csr* pins, const dr_csr* pinned,
                      int32_t D, int32_t k_cell, int32_t k_net) {
    return heteroconv_create_widths(ctx, near, pins, pinned, D, k_cell, k_cell, k_net, k_net);
}

int heteroconv_create_per_relation(dr_heteroconv** ctx, const dr_csr* near, const dr_csr* pins, const dr_csr* pinned,
                                   int32_t D, int32_t k_near, int32_t k_pins, int32_t k_pinned) {
    return heteroconv_create_widths(ctx, near, pins, pinned, D, k_near, k_pins, k_pins, k_pinned);
}

int heteroconv_get_k(const dr_heteroconv* ctx, int32_t* k_near, int32_t* k_pins, int32_t* k_self, int32_t* k_pinned) {
    DRC_REQUIRE(ctx && k_near && k_pins && k_self && k_pinned, "heteroconv_get_k: null argument");
    *k_near = ctx->k_near; *k_pins = ctx->k_pins; *k_self = ctx->k_self; *k_pinned = ctx->k_pinned;
    return DR_OK;
}

int heteroconv_destroy(dr_heteroconv* ctx) {
    if (!ctx) return DR_OK;
    (void)hipDeviceSynchronize();
    release(ctx);
    return DR_OK;
}

int heteroconv_get_transpose(const dr_heteroconv* ctx, int which, dr_csr* out) {
    DRC_REQUIRE(ctx && out, "heteroconv_get_transpose: null argument");
    DRC_REQUIRE(which >= 0 && which < 3, "heteroconv_get_transpose: which must be 0, 1 or 2");
    *out = ctx->At[which];
    return DR_OK;
}

int heteroconv_set_cell_order(dr_heteroconv* ctx, const int32_t* cell_order, int* staged, void* stream) {
    DRC_REQUIRE(ctx != nullptr, "heteroconv_set_cell_order: null context");
    if (staged) *staged = 0;
    if (ctx->near_plan) {
        DRC_HIP(hipDeviceSynchronize());      // work that still reads the old plan
        spmm_plan_destroy(ctx->near_plan);
        ctx->near_plan = nullptr;
    }
    if (ctx->At[0].nnz == 0) return DR_OK;
    const int cw = ctx->D % 64 == 0 ? 64 : 32;
    if (ctx->D % 32 != 0 || ctx->D / cw > 4 || ctx->k_near > 2 * cw) return DR_OK;      // widths the staged kernel does not cover
    dr_spmm_plan* plan = nullptr;
    const int rc = spmm_plan_create(&plan, &ctx->At[0], cell_order, ctx->D, as_stream(stream));
    if (rc == DR_ERR_UNSUPPORTED) return DR_OK;        // a row that does not fit a tile: the plain kernel stays
    if (rc != DR_OK) return rc;
    int64_t n_tiles = 0;
    double reuse = 0.0;
    DRC_TRY(dr_spmm_plan_info(plan, &n_tiles, &reuse));
    if (reuse < kMinStagingReuse) {                    // nothing to gain from staging: rows of a tile share too few neighbours
        spmm_plan_destroy(plan);
        return DR_OK;
    }
    ctx->near_plan = plan;
    if (staged) *staged = 1;
    return DR_OK;
}

int heteroconv_set_overlap(dr_heteroconv* ctx, int mode) {
    DRC_REQUIRE(ctx != nullptr, "heteroconv_set_overlap: null context");
    DRC_REQUIRE(mode == DR_OVERLAP_AUTO || mode == DR_OVERLAP_ON || mode == DR_OVERLAP_OFF,
                "heteroconv_set_overlap: unknown mode %d", mode);
    ctx->overlap = mode;
    return DR_OK;
}

// Separate streams pay off while one relation's kernels leave CUs idle at their tails (measured on MI355X:
// 1.6x on 60k-cell graphs, 1.15x at 250k cells).  At 1.2M cells every launch has tens of thousands of
// workgroups and the three pipelines only time-slice the CUs (1.5% difference), so they are issued back to
// back on one stream instead, which keeps per-kernel timings attributable.
static bool relations_overlap(const dr_heteroconv* c) {
    if (c->overlap == DR_OVERLAP_ON) return true;
    if (c->overlap == DR_OVERLAP_OFF) return false;
    const int64_t rows = c->Nc > c->Nn ? c->Nc : c->Nn;
    return rows * c->D < (int64_t(1) << 26);
}

int heteroconv_profile(dr_heteroconv* ctx, int enable) {
    DRC_REQUIRE(ctx != nullptr, "heteroconv_profile: null context");
    DRC_REQUIRE(ctx->timed && ctx->event_pool, "heteroconv_profile: out of host memory");
    ctx->profile = enable != 0;
    return DR_OK;
}

int heteroconv_profile_k(dr_heteroconv* c, const float* X_cell, const float* X_net, const int32_t* candidates,
                         int32_t n_candidates, int32_t warmup, int32_t reps, float* ms_fwd, float* ms_bwd,
                         int32_t* best_k) {
    DRC_REQUIRE(c != nullptr, "heteroconv_profile_k: null context");
    DRC_REQUIRE(X_cell && X_net && candidates && ms_fwd && ms_bwd && best_k, "heteroconv_profile_k: null argument");
    DRC_REQUIRE(aligned(X_cell, 16) && aligned(X_net, 16), "heteroconv_profile_k: embeddings must be 16-byte aligned");
    DRC_REQUIRE(n_candidates >= 1 && n_candidates <= 64, "heteroconv_profile_k: n_candidates = %d out of range [1, 64]", n_candidates);
    DRC_REQUIRE(warmup >= 0 && reps >= 1 && reps <= 1000, "heteroconv_profile_k: warmup = %d, reps = %d", warmup, reps);
    int kmax = 0;
    for (int i = 0; i < n_candidates; ++i) {
        DRC_REQUIRE(candidates[i] >= 1 && candidates[i] <= c->D, "heteroconv_profile_k: candidate %d is %d, D = %d", i,
                    candidates[i], c->D);
        if (candidates[i] > kmax) kmax = candidates[i];
    }
    const int D = c->D;
    const size_t rows = (size_t)(c->Nc > c->Nn ? c->Nc : c->Nn);
    float *vals = nullptr, *H = nullptr, *G = nullptr;
    uint16_t* idx = nullptr;
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    hipStream_t s = c->st[0];
    auto body = [&]() -> int {
        DRC_HIP(hipDeviceSynchronize());
        DRC_HIP(hipMalloc((void**)&vals, 4 * rows * kmax + 256));
        DRC_HIP(hipMalloc((void**)&idx, 2 * rows * kmax + 256));
        DRC_HIP(hipMalloc((void**)&G, 4 * rows * kmax + 256));
        DRC_HIP(hipMalloc((void**)&H, 4 * rows * D + 256));
        for (hipEvent_t& e : ev) DRC_HIP(hipEventCreate(&e));
        for (int r = 0; r < 3; ++r) {
            // sources of near and pins are cells, of pinned nets; the upstream gradient of the backward is any
            // dense [M, D] array (the kernels' time does not depend on values): the destination type's embeddings
            const float* Xsrc = (r == 2) ? X_net : X_cell;
            const float* dH = (r == 1) ? X_net : X_cell;
            const int64_t n_src = c->A[r].n_cols;
            int best = -1;
            float best_ms = 0.f;
            for (int i = 0; i < n_candidates; ++i) {
                const int k = candidates[i];
                DRC_TRY(launch_topk(Xsrc, n_src, D, k, vals, idx, s));
                for (int w = 0; w < warmup; ++w) {
                    DRC_TRY(launch_spmm_fwd(&c->A[r], vals, idx, D, k, H, s));
                    DRC_TRY(launch_spmm_bwd(&c->At[r], dH, idx, D, k, G, 0, s));
                }
                DRC_HIP(hipEventRecord(ev[0], s));
                for (int q = 0; q < reps; ++q) DRC_TRY(launch_spmm_fwd(&c->A[r], vals, idx, D, k, H, s));
                DRC_HIP(hipEventRecord(ev[1], s));
                for (int q = 0; q < reps; ++q) DRC_TRY(launch_spmm_bwd(&c->At[r], dH, idx, D, k, G, 0, s));
                DRC_HIP(hipEventRecord(ev[2], s));
                DRC_HIP(hipEventSynchronize(ev[2]));
                float f = 0.f, b = 0.f;
                DRC_HIP(hipEventElapsedTime(&f, ev[0], ev[1]));
                DRC_HIP(hipEventElapsedTime(&b, ev[1], ev[2]));
                ms_fwd[r * n_candidates + i] = f / reps;
                ms_bwd[r * n_candidates + i] = b / reps;
                const float tot = (f + b) / reps;
                if (best < 0 || tot < best_ms || (tot == best_ms && k < candidates[best])) { best = i; best_ms = tot; }
            }
            best_k[r] = candidates[best];
        }
        return DR_OK;
    };
    const int rc = body();
    (void)hipDeviceSynchronize();
    for (hipEvent_t e : ev)
        if (e) (void)hipEventDestroy(e);
    (void)hipFree(vals); (void)hipFree(idx); (void)hipFree(G); (void)hipFree(H);
    return rc;
}

int heteroconv_num_kernels(void) { return kNumKernels; }

const char* heteroconv_kernel_name(int id) { return (id >= 0 && id < kNumKernels) ? kKernelNames[id] : ""; }

int heteroconv_kernel_times(dr_heteroconv* ctx, double* ms_sum, int64_t* launches, int n) {
    DRC_REQUIRE(ctx && ms_sum && launches, "heteroconv_kernel_times: null argument");
    DRC_REQUIRE(n >= kNumKernels, "heteroconv_kernel_times: arrays need heteroconv_num_kernels() entries");
    for (int i = 0; i < n; ++i) { ms_sum[i] = 0.0; launches[i] = 0; }
    DRC_HIP(hipDeviceSynchronize());
    for (TimedLaunch& t : *ctx->timed) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, t.start, t.stop) == hipSuccess) { ms_sum[t.id] += ms; launches[t.id] += 1; }
        if (!t.start_shared) ctx->event_pool->push_back(t.start);
        ctx->event_pool->push_back(t.stop);
    }
    ctx->timed->clear();
    return DR_OK;
}

static int check_weights(const dr_heteroconv_weights* W, const char* fn) {
    DRC_REQUIRE(W != nullptr, "%s: null weights", fn);
    DRC_REQUIRE(W->self_near && W->neigh_near && W->self_pins && W->neigh_pins && W->pinned,
                "%s: null weight matrix", fn);
    DRC_REQUIRE(aligned(W->self_near, 16) && aligned(W->neigh_near, 16) && aligned(W->self_pins, 16) &&
                    aligned(W->neigh_pins, 16) && aligned(W->pinned, 16),
                "%s: weight matrices must be 16-byte aligned", fn);
    return DR_OK;
}

static int check_saved(const dr_heteroconv* c, const dr_heteroconv_saved* S, const char* fn) {
    DRC_REQUIRE(S != nullptr, "%s: null saved", fn);
    DRC_REQUIRE(S->vals_cell && S->idx_cell && S->vals_net && S->idx_net && S->H_near && S->H_pins &&
                    S->H_pinned && S->mask,
                "%s: null buffer in saved", fn);
    DRC_REQUIRE(aligned(S->H_near, 16) && aligned(S->H_pins, 16) && aligned(S->H_pinned, 16) &&
                    aligned(S->mask, 4) && aligned(S->vals_cell, 4) && aligned(S->vals_net, 4),
                "%s: misaligned buffer in saved", fn);
    if (c->k_pins != c->k_near)
        DRC_REQUIRE(S->vals_cell_pins && S->idx_cell_pins && aligned(S->vals_cell_pins, 4),
                    "%s: k_pins != k_near needs saved.vals_cell_pins / idx_cell_pins", fn);
    if (c->k_self != c->k_pinned)
        DRC_REQUIRE(S->vals_net_self && S->idx_net_self && aligned(S->vals_net_self, 4),
                    "%s: k_pins != k_pinned needs saved.vals_net_self / idx_net_self", fn);
    return DR_OK;
}

// The CBSR each use of an embedding reads: a width shared by both uses of a node type shares the buffers.
struct CbsrSets {
    const float *v_near, *v_pins, *v_self, *v_pinned;
    const uint16_t *i_near, *i_pins, *i_self, *i_pinned;
    bool cell_split, net_split;
};
static CbsrSets cbsr_sets(const dr_heteroconv* c, const dr_heteroconv_saved* S) {
    CbsrSets q;
    q.cell_split = c->k_pins != c->k_near;
    q.net_split = c->k_self != c->k_pinned;
    q.v_near = S->vals_cell; q.i_near = S->idx_cell;
    q.v_pinned = S->vals_net; q.i_pinned = S->idx_net;
    q.v_pins = q.cell_split ? S->vals_cell_pins : S->vals_cell;
    q.i_pins = q.cell_split ? S->idx_cell_pins : S->idx_cell;
    q.v_self = q.net_split ? S->vals_net_self : S->vals_net;
    q.i_self = q.net_split ? S->idx_net_self : S->idx_net;
    return q;
}

int heteroconv_fwd(dr_heteroconv* c, const float* X_cell, const float* X_net, const dr_heteroconv_weights* W,
                   float* Y_cell, float* Y_net, const dr_heteroconv_saved* S, void* stream) {
    return heteroconv_forward(c, X_cell, X_net, W, Y_cell, Y_net, S, stream, ForwardOptions{});
}

int heteroconv_bwd(dr_heteroconv* c, const float* dY_cell, const float* dY_net, const dr_heteroconv_weights* W,
                   const dr_heteroconv_saved* S, float* dX_cell, float* dX_net, const dr_heteroconv_wgrads* dW,
                   void* stream) {
    return heteroconv_backward(c, dY_cell, dY_net, W, S, dX_cell, dX_net, dW, stream, BackwardOptions{});
}

}  // extern "C"

int drc::heteroconv_forward(dr_heteroconv* c, const float* X_cell, const float* X_net, const dr_heteroconv_weights* W,
                            float* Y_cell, float* Y_net, const dr_heteroconv_saved* S, void* stream, ForwardOptions opt) {
    // opt.skip_net_output: Y_net is not wanted (last layer of a model whose read-out uses the cells only): the pins
    // module -- its DR-SpMM and its projection -- is not launched, and H_pins / Y_net are left untouched.
    const bool relu_out = opt.relu_out, pins_module = !opt.skip_net_output;
    DRC_REQUIRE(c != nullptr, "heteroconv_fwd: null context");
    DRC_REQUIRE(X_cell && X_net && Y_cell && Y_net, "heteroconv_fwd: null tensor");
    DRC_REQUIRE(aligned(X_cell, 16) && aligned(X_net, 16) && aligned(Y_cell, 16) && aligned(Y_net, 16),
                "heteroconv_fwd: tensors must be 16-byte aligned");
    DRC_TRY(check_weights(W, "heteroconv_fwd"));
    DRC_TRY(check_saved(c, S, "heteroconv_fwd"));
    hipStream_t user = as_stream(stream);
    const bool ov = relations_overlap(c);
    hipStream_t s_near = c->st[0], s_pins = ov ? c->st[1] : c->st[0], s_pinned = ov ? c->st[2] : c->st[0];
    c->chain_stop = nullptr; c->chain_ok = !ov;
    const int D = c->D;

    DRC_HIP(hipEventRecord(c->ev_fork, user));
    for (int i = 0; i < (ov ? 3 : 1); ++i) DRC_HIP(hipStreamWaitEvent(c->st[i], c->ev_fork, 0));   // only the streams that get work

    // Enqueue order (it is the execution order when all relations share one stream): every D-ReLU output is
    // gathered right after it is written, while it is still resident in the memory-side cache; the random
    // relations (pinned, pins) come before the grid-local one, and the streaming projections last.
    const CbsrSets q = cbsr_sets(c, S);

    // D-ReLU(net), then pinned: net -> cell.  A node type that is read at two widths is selected at both in one
    // pass over its embeddings.
    {
        ScopedTiming tm(c, kTopkNet, s_pinned);
        DRC_TRY(launch_topk2(X_net, c->Nn, D, c->k_pinned, S->vals_net, S->idx_net, c->k_self,
                             q.net_split ? S->vals_net_self : nullptr, q.net_split ? S->idx_net_self : nullptr, s_pinned));
    }
    DRC_HIP(hipEventRecord(c->ev_topk_net, s_pinned));
    { ScopedTiming tm(c, kFwdPinned, s_pinned); DRC_TRY(launch_spmm_fwd(&c->A[2], q.v_pinned, q.i_pinned, D, c->k_pinned, S->H_pinned, s_pinned)); }

    // D-ReLU(cell), then pins: cell -> net and near: cell -> cell
    {
        ScopedTiming tm(c, kTopkCell, s_near);
        DRC_TRY(launch_topk2(X_cell, c->Nc, D, c->k_near, S->vals_cell, S->idx_cell, c->k_pins,
                             q.cell_split ? S->vals_cell_pins : nullptr, q.cell_split ? S->idx_cell_pins : nullptr, s_near));
    }
    DRC_HIP(hipEventRecord(c->ev_topk_cell, s_near));
    DRC_HIP(hipStreamWaitEvent(s_pins, c->ev_topk_cell, 0));
    if (pins_module) { ScopedTiming tm(c, kFwdPins, s_pins); DRC_TRY(launch_spmm_fwd(&c->A[1], q.v_pins, q.i_pins, D, c->k_pins, S->H_pins, s_pins)); }
    { ScopedTiming tm(c, kFwdNear, s_near); DRC_TRY(launch_spmm_fwd(&c->A[0], q.v_near, q.i_near, D, c->k_near, S->H_near, s_near)); }

    // projections: near (self + neighbour), pins (self + neighbour), pinned merged into Y_cell by max
    {
        GemmOperand seg[2] = {};
        seg[0].cbsr_vals = q.v_near; seg[0].cbsr_idx = q.i_near; seg[0].k = c->k_near; seg[0].W = W->self_near;
        seg[1].dense = S->H_near; seg[1].W = W->neigh_near;
        { ScopedTiming tm(c, kProjNear, s_near); DRC_TRY(launch_gemm(seg, 2, c->Nc, D, kEpiStore, Y_cell, nullptr, SampleSet{}, SampleSet{}, s_near)); }
    }
    DRC_HIP(hipEventRecord(c->ev_near, s_near));
    DRC_HIP(hipStreamWaitEvent(s_pins, c->ev_topk_net, 0));
    if (pins_module) {
        GemmOperand seg[2] = {};
        seg[0].cbsr_vals = q.v_self; seg[0].cbsr_idx = q.i_self; seg[0].k = c->k_self; seg[0].W = W->self_pins;
        seg[1].dense = S->H_pins; seg[1].W = W->neigh_pins;
        { ScopedTiming tm(c, kProjPins, s_pins); DRC_TRY(launch_gemm(seg, 2, c->Nn, D, kEpiStore, Y_net, nullptr, SampleSet{}, SampleSet{}, s_pins, relu_out ? 1 : 0)); }
    }
    DRC_HIP(hipEventRecord(c->ev_pins, s_pins));
    DRC_HIP(hipStreamWaitEvent(s_pinned, c->ev_near, 0));
    {
        GemmOperand seg[1] = {};
        seg[0].dense = S->H_pinned; seg[0].W = W->pinned;
        { ScopedTiming tm(c, kProjPinnedMerge, s_pinned); DRC_TRY(launch_gemm(seg, 1, c->Nc, D, kEpiMaxMerge, Y_cell, S->mask, SampleSet{}, SampleSet{}, s_pinned, relu_out ? 1 : 0)); }
    }
    DRC_HIP(hipEventRecord(c->ev_pinned, s_pinned));

    DRC_HIP(hipStreamWaitEvent(user, c->ev_pins, 0));
    DRC_HIP(hipStreamWaitEvent(user, c->ev_pinned, 0));
    return DR_OK;
}

int drc::heteroconv_backward(dr_heteroconv* c, const float* dY_cell, const float* dY_net, const dr_heteroconv_weights* W,
                             const dr_heteroconv_saved* S, float* dX_cell, float* dX_net, const dr_heteroconv_wgrads* dW,
                             void* stream, BackwardOptions opt) {
    // opt.skip_dx: only the weight gradients are wanted (first layer of a model: nobody reads the gradient of the
    // input features), so the projections to dH, the transposed SpMMs and the dX write-outs are not launched.
    // opt.dy_net_zero: dY_net holds zeros (last layer of a model whose loss reads the cells only): everything it
    // would feed is zero, so the pins module's dH, transposed SpMM and weight-gradient kernels are replaced by fills.
    const bool gate_inputs = opt.gate_inputs, need_dx = !opt.skip_dx, net_zero = opt.dy_net_zero;
    DRC_REQUIRE(c != nullptr, "heteroconv_bwd: null context");
    DRC_REQUIRE(dY_cell && dY_net && (!need_dx || (dX_cell && dX_net)), "heteroconv_bwd: null tensor");
    DRC_REQUIRE(aligned(dY_cell, 16) && aligned(dY_net, 16) && aligned(dX_cell, 16) && aligned(dX_net, 16),
                "heteroconv_bwd: misaligned tensor");
    DRC_TRY(check_weights(W, "heteroconv_bwd"));
    DRC_TRY(check_saved(c, S, "heteroconv_bwd"));
    DRC_REQUIRE(dW && dW->self_near && dW->neigh_near && dW->self_pins && dW->neigh_pins && dW->pinned,
                "heteroconv_bwd: null weight gradient");
    hipStream_t user = as_stream(stream);
    const bool ov = relations_overlap(c);
    hipStream_t s_near = c->st[0], s_pins = ov ? c->st[1] : c->st[0], s_pinned = ov ? c->st[2] : c->st[0];
    c->chain_stop = nullptr; c->chain_ok = !ov;
    const int D = c->D;

    DRC_HIP(hipEventRecord(c->ev_fork, user));
    for (int i = 0; i < (ov ? 3 : 1); ++i) DRC_HIP(hipStreamWaitEvent(c->st[i], c->ev_fork, 0));   // only the streams that get work

    const CbsrSets q = cbsr_sets(c, S);

    // ---- near stream: dH_near, its transposed SpMM (first piece of dXs_cell), near weight gradients ----
    if (need_dx) {
        GemmOperand seg[1] = {};
        seg[0].dense = dY_cell; seg[0].mask = S->mask; seg[0].mask_keep = 1;
        seg[0].W = W->neigh_near; seg[0].transpose_w = 1;
        { ScopedTiming tm(c, kDhNear, s_near); DRC_TRY(launch_gemm(seg, 1, c->Nc, D, kEpiStore, c->dH[0], nullptr, SampleSet{}, SampleSet{}, s_near)); }
        {
            ScopedTiming tm(c, kBwdNear, s_near);
            if (c->near_plan) DRC_TRY(launch_spmm_bwd_planned(c->near_plan, c->dH[0], q.i_near, c->k_near, c->dXs_cell, 0, s_near));
            else DRC_TRY(launch_spmm_bwd(&c->At[0], c->dH[0], q.i_near, D, c->k_near, c->dXs_cell, 0, s_near));
        }
        DRC_HIP(hipEventRecord(c->ev_gnear, s_near));
    }
    {
        // both near weight gradients share dZ_near: one pass forms H_near^T dZ and Xs_cell^T dZ together
        WgradOperand op = {};
        op.a_dense = S->H_near; op.a_cbsr_vals = q.v_near; op.a_cbsr_idx = q.i_near; op.k = c->k_near;
        op.b = dY_cell; op.b_mask = S->mask; op.b_mask_keep = 1;
        { ScopedTiming tm(c, kWgNear, s_near); DRC_TRY(launch_wgrad(op, c->Nc, D, dW->neigh_near, dW->self_near, c->wg_scratch[0], s_near)); }
    }
    DRC_HIP(hipEventRecord(c->ev_near, s_near));

    // ---- pins stream: dH_pins, second piece of the cell gradient, near self term, dense dX_cell, pins weight gradients.
    // With one width for the cells the pins piece is added into dXs_cell; with two it keeps its own buffer and
    // the write-out kernel adds it at its own positions. ----
    const bool pins_piece = need_dx && !net_zero;           // the pins module's contribution to the cell gradient
    if (pins_piece) {
        GemmOperand seg[1] = {};
        seg[0].dense = dY_net; seg[0].W = W->neigh_pins; seg[0].transpose_w = 1;
        { ScopedTiming tm(c, kDhPins, s_pins); DRC_TRY(launch_gemm(seg, 1, c->Nn, D, kEpiStore, c->dH[1], nullptr, SampleSet{}, SampleSet{}, s_pins)); }
        if (!q.cell_split) DRC_HIP(hipStreamWaitEvent(s_pins, c->ev_gnear, 0));
        { ScopedTiming tm(c, kBwdPins, s_pins); DRC_TRY(launch_spmm_bwd(&c->At[1], c->dH[1], q.i_pins, D, c->k_pins, q.cell_split ? c->dXs_cell_b : c->dXs_cell,
                                                                        q.cell_split ? 0 : 1, s_pins)); }
    }
    if (need_dx) {
        if (q.cell_split || !pins_piece) DRC_HIP(hipStreamWaitEvent(s_pins, c->ev_gnear, 0));
        GemmOperand seg[1] = {};
        seg[0].dense = dY_cell; seg[0].mask = S->mask; seg[0].mask_keep = 1;
        seg[0].W = W->self_near; seg[0].transpose_w = 1;
        const SampleSet first{q.i_near, c->k_near, c->dXs_cell, gate_inputs ? q.v_near : nullptr};
        const SampleSet second = (q.cell_split && pins_piece) ? SampleSet{q.i_pins, c->k_pins, c->dXs_cell_b, gate_inputs ? q.v_pins : nullptr}
                                                             : SampleSet{};
        { ScopedTiming tm(c, kSelfNearSample, s_pins); DRC_TRY(launch_gemm(seg, 1, c->Nc, D, kEpiSampleDense, dX_cell, nullptr, first, second, s_pins)); }
    }
    if (net_zero) {
        DRC_TRY(launch_fill_u32(reinterpret_cast<uint32_t*>(dW->neigh_pins), (size_t)D * D, 0u, s_pins));
        DRC_TRY(launch_fill_u32(reinterpret_cast<uint32_t*>(dW->self_pins), (size_t)D * D, 0u, s_pins));
    } else {
        WgradOperand op = {};
        op.a_dense = S->H_pins; op.a_cbsr_vals = q.v_self; op.a_cbsr_idx = q.i_self; op.k = c->k_self; op.b = dY_net;
        { ScopedTiming tm(c, kWgPins, s_pins); DRC_TRY(launch_wgrad(op, c->Nn, D, dW->neigh_pins, dW->self_pins, c->wg_scratch[1], s_pins)); }
    }
    DRC_HIP(hipEventRecord(c->ev_pins, s_pins));

    // ---- pinned stream: dH_pinned, dXs_net, pins self term, dense dX_net, pinned weight gradient.  With two widths
    // for the nets the self term is sampled at its own selection and the pinned piece added at the other. ----
    if (need_dx) {
        GemmOperand seg[1] = {};
        seg[0].dense = dY_cell; seg[0].mask = S->mask; seg[0].mask_keep = 0;
        seg[0].W = W->pinned; seg[0].transpose_w = 1;
        { ScopedTiming tm(c, kDhPinned, s_pinned); DRC_TRY(launch_gemm(seg, 1, c->Nc, D, kEpiStore, c->dH[2], nullptr, SampleSet{}, SampleSet{}, s_pinned)); }
        { ScopedTiming tm(c, kBwdPinned, s_pinned); DRC_TRY(launch_spmm_bwd(&c->At[2], c->dH[2], q.i_pinned, D, c->k_pinned, c->dXs_net, 0, s_pinned)); }
        GemmOperand sg[1] = {};
        sg[0].dense = dY_net; sg[0].W = W->self_pins; sg[0].transpose_w = 1;
        const float* g_self = gate_inputs ? q.v_self : nullptr;
        const float* g_pinned = gate_inputs ? q.v_pinned : nullptr;
        const SampleSet first = q.net_split ? SampleSet{q.i_self, c->k_self, nullptr, g_self} : SampleSet{q.i_pinned, c->k_pinned, c->dXs_net, g_pinned};
        const SampleSet second = q.net_split ? SampleSet{q.i_pinned, c->k_pinned, c->dXs_net, g_pinned} : SampleSet{};
        { ScopedTiming tm(c, kSelfPinsSample, s_pinned); DRC_TRY(launch_gemm(sg, 1, c->Nn, D, kEpiSampleDense, dX_net, nullptr, first, second, s_pinned)); }
    }
    {
        WgradOperand op = {};
        op.a_dense = S->H_pinned; op.b = dY_cell; op.b_mask = S->mask; op.b_mask_keep = 0;
        { ScopedTiming tm(c, kWgPinned, s_pinned); DRC_TRY(launch_wgrad(op, c->Nc, D, dW->pinned, nullptr, c->wg_scratch[2], s_pinned)); }
    }
    DRC_HIP(hipEventRecord(c->ev_pinned, s_pinned));

    DRC_HIP(hipStreamWaitEvent(user, c->ev_near, 0));
    DRC_HIP(hipStreamWaitEvent(user, c->ev_pins, 0));
    DRC_HIP(hipStreamWaitEvent(user, c->ev_pinned, 0));
    return DR_OK;
}
