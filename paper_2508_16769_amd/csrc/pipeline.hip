// Host-side pipeline (paper Section 3.4 and the breakdown in Section 4.4: data loading, initialisation and the
// host-to-device copies of the next sub-graphs run on CPU threads and their own streams while the GPU works on the
// current ones).  A pipeline owns a few SLOTS.  A slot has pinned staging memory, device arrays sized for the
// largest graph it will see, a re-bindable layer context and a stream.  dr_pipeline_submit hands a host graph to
// a worker thread, which
//   1. waits (on the host, in the worker) until the GPU is done with the slot's previous graph,
//   2. copies the caller's arrays into the slot's pinned staging memory (so the upload is a true async copy),
//   3. enqueues on the slot's stream: the uploads, the pinned pattern (= transpose of pins), the edge values of
//      the three modules, and the three transposed adjacencies of the layer context,
//   4. records the slot's `ready` event.
// dr_pipeline_acquire waits for step 4 to have been ENQUEUED and makes the caller's stream wait for the event:
// the host never waits for the GPU on the consumer side, and nothing here allocates after dr_pipeline_create.
#include "dr_internal.h"

#include <condition_variable>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

namespace {

using namespace drc;

enum SlotState { kIdle = 0, kQueued = 1, kReady = 2, kAcquired = 3, kFailed = 4 };

struct Slot {
    // device arrays at capacity
    int32_t *near_rp, *near_ci, *pins_rp, *pins_ci, *pinned_rp, *pinned_ci;
    float *near_v, *pins_v, *pinned_v;
    float *X_cell, *X_net;
    void *ws_t, *ws_n;
    size_t ws_t_bytes, ws_n_bytes;
    // pinned staging: near_rp | near_ci | pins_rp | pins_ci | X_cell | X_net
    char* stage;
    size_t off_near_ci, off_pins_rp, off_pins_ci, off_xc, off_xn, stage_bytes;
    dr_heteroconv* ctx;
    dr_csr rel[3];
    hipStream_t stream;
    hipEvent_t ready, freed;
    bool freed_pending;
    int state;
    int rc;
    std::string err;
    dr_host_graph job;
};

}  // namespace

struct dr_pipeline {
    std::vector<Slot> slots;
    std::vector<std::thread> workers;
    std::mutex mu;
    std::condition_variable cv_job, cv_done;
    std::deque<int> queue;
    bool stop;
    int device, D;
    int64_t cap_cells, cap_nets, cap_near, cap_pins;
    std::vector<void*> dev_mem, host_mem;
};

namespace {

size_t up256(size_t b) { return (b + 255) & ~size_t(255); }

int process(dr_pipeline* p, Slot& s) {
    const dr_host_graph& g = s.job;
    const int D = p->D;
    if (s.freed_pending) {                      // the GPU may still be working on the slot's previous graph
        DRC_HIP(hipEventSynchronize(s.freed));
        s.freed_pending = false;
    }
    const size_t n_rp = 4 * (size_t)(g.n_cells + 1), n_ci = 4 * (size_t)g.nnz_near;
    const size_t p_rp = 4 * (size_t)(g.n_nets + 1), p_ci = 4 * (size_t)g.nnz_pins;
    const size_t xc = g.X_cell ? 4 * (size_t)g.n_cells * D : 0, xn = g.X_net ? 4 * (size_t)g.n_nets * D : 0;
    std::memcpy(s.stage, g.near_rowptr, n_rp);
    if (n_ci) std::memcpy(s.stage + s.off_near_ci, g.near_colidx, n_ci);
    std::memcpy(s.stage + s.off_pins_rp, g.pins_rowptr, p_rp);
    if (p_ci) std::memcpy(s.stage + s.off_pins_ci, g.pins_colidx, p_ci);
    if (xc) std::memcpy(s.stage + s.off_xc, g.X_cell, xc);
    if (xn) std::memcpy(s.stage + s.off_xn, g.X_net, xn);
    hipStream_t st = s.stream;
    DRC_HIP(hipMemcpyAsync(s.near_rp, s.stage, n_rp, hipMemcpyHostToDevice, st));
    if (n_ci) DRC_HIP(hipMemcpyAsync(s.near_ci, s.stage + s.off_near_ci, n_ci, hipMemcpyHostToDevice, st));
    DRC_HIP(hipMemcpyAsync(s.pins_rp, s.stage + s.off_pins_rp, p_rp, hipMemcpyHostToDevice, st));
    if (p_ci) DRC_HIP(hipMemcpyAsync(s.pins_ci, s.stage + s.off_pins_ci, p_ci, hipMemcpyHostToDevice, st));
    if (xc) DRC_HIP(hipMemcpyAsync(s.X_cell, s.stage + s.off_xc, xc, hipMemcpyHostToDevice, st));
    if (xn) DRC_HIP(hipMemcpyAsync(s.X_net, s.stage + s.off_xn, xn, hipMemcpyHostToDevice, st));
    // pinned pattern = transpose of the pins pattern
    dr_csr pins_pat{g.n_nets, g.n_cells, g.nnz_pins, s.pins_rp, s.pins_ci, nullptr};
    DRC_TRY(dr_csr_transpose(&pins_pat, s.pinned_rp, s.pinned_ci, nullptr, s.ws_t, s.ws_t_bytes, st));
    // edge values of the three modules
    DRC_TRY(dr_csr_normalize(DR_NORM_MEAN, g.n_cells, g.n_cells, g.nnz_near, s.near_rp, s.near_ci, s.near_v, s.ws_n, s.ws_n_bytes, st));
    DRC_TRY(dr_csr_normalize(DR_NORM_MEAN, g.n_nets, g.n_cells, g.nnz_pins, s.pins_rp, s.pins_ci, s.pins_v, s.ws_n, s.ws_n_bytes, st));
    DRC_TRY(dr_csr_normalize(DR_NORM_SYM, g.n_cells, g.n_nets, g.nnz_pins, s.pinned_rp, s.pinned_ci, s.pinned_v, s.ws_n, s.ws_n_bytes, st));
    s.rel[0] = dr_csr{g.n_cells, g.n_cells, g.nnz_near, s.near_rp, s.near_ci, s.near_v};
    s.rel[1] = dr_csr{g.n_nets, g.n_cells, g.nnz_pins, s.pins_rp, s.pins_ci, s.pins_v};
    s.rel[2] = dr_csr{g.n_cells, g.n_nets, g.nnz_pins, s.pinned_rp, s.pinned_ci, s.pinned_v};
    DRC_TRY(heteroconv_bind(s.ctx, &s.rel[0], &s.rel[1], &s.rel[2], st));
    DRC_HIP(hipEventRecord(s.ready, st));
    return DR_OK;
}

void worker_main(dr_pipeline* p) {
    const bool dev_ok = hipSetDevice(p->device) == hipSuccess;
    for (;;) {
        int id;
        {
            std::unique_lock<std::mutex> lk(p->mu);
            p->cv_job.wait(lk, [&] { return p->stop || !p->queue.empty(); });
            if (p->queue.empty()) return;          // stop requested and nothing left to do
            id = p->queue.front();
            p->queue.pop_front();
        }
        Slot& s = p->slots[id];
        int rc = dev_ok ? process(p, s) : DR_ERR_HIP;
        std::string err = rc == DR_OK ? std::string() : (dev_ok ? std::string(dr_last_error()) : std::string("hipSetDevice failed in a worker thread"));
        {
            std::lock_guard<std::mutex> lk(p->mu);
            s.rc = rc;
            s.err = err;
            s.state = rc == DR_OK ? kReady : kFailed;
        }
        p->cv_done.notify_all();
    }
}

int dev_alloc(std::vector<void*>& owned, void** ptr, size_t bytes) {
    *ptr = nullptr;
    DRC_HIP(hipMalloc(ptr, bytes ? bytes : 256));
    owned.push_back(*ptr);
    return DR_OK;
}

}  // namespace

extern "C" {

int dr_pipeline_destroy(dr_pipeline* p) {
    if (!p) return DR_OK;
    {
        std::lock_guard<std::mutex> lk(p->mu);
        p->stop = true;
    }
    p->cv_job.notify_all();
    for (auto& t : p->workers) t.join();
    (void)hipDeviceSynchronize();
    for (Slot& s : p->slots) {
        if (s.ctx) (void)heteroconv_destroy(s.ctx);
        if (s.stream) (void)hipStreamDestroy(s.stream);
        if (s.ready) (void)hipEventDestroy(s.ready);
        if (s.freed) (void)hipEventDestroy(s.freed);
    }
    for (void* d : p->dev_mem) (void)hipFree(d);
    for (void* h : p->host_mem) (void)hipHostFree(h);
    delete p;
    return DR_OK;
}

int dr_pipeline_create(dr_pipeline** out, int32_t n_slots, int32_t n_threads, int64_t max_cells, int64_t max_nets,
                       int64_t max_nnz_near, int64_t max_nnz_pins, int32_t D, int32_t k_cell, int32_t k_net) {
    DRC_REQUIRE(out != nullptr, "dr_pipeline_create: null out");
    *out = nullptr;
    DRC_REQUIRE(n_slots >= 1 && n_slots <= 64, "dr_pipeline_create: n_slots = %d out of range [1, 64]", n_slots);
    DRC_REQUIRE(n_threads >= 1 && n_threads <= 16, "dr_pipeline_create: n_threads = %d out of range [1, 16]", n_threads);
    DRC_REQUIRE(max_cells >= 1 && max_nets >= 1 && max_nnz_near >= 0 && max_nnz_pins >= 0, "dr_pipeline_create: bad capacity");
    DRC_REQUIRE(max_nnz_near < (int64_t(1) << 31) && max_nnz_pins < (int64_t(1) << 31), "dr_pipeline_create: nnz >= 2^31");
    dr_pipeline* p = new (std::nothrow) dr_pipeline();
    if (!p) return fail(DR_ERR_HIP, "dr_pipeline_create: out of host memory");
    p->stop = false; p->D = D;
    p->cap_cells = max_cells; p->cap_nets = max_nets; p->cap_near = max_nnz_near; p->cap_pins = max_nnz_pins;
    p->slots.resize(n_slots);
    for (Slot& s : p->slots) {
        s = Slot{};
        s.state = kIdle;
    }
    auto body = [&]() -> int {
        DRC_HIP(hipGetDevice(&p->device));
        const int64_t E[3] = {max_nnz_near, max_nnz_pins, max_nnz_pins};
        for (Slot& s : p->slots) {
            DRC_TRY(dev_alloc(p->dev_mem, (void**)&s.near_rp, 4 * (size_t)(max_cells + 1)));
            DRC_TRY(dev_alloc(p->dev_mem, (void**)&s.near_ci, 4 * (size_t)max_nnz_near));
            DRC_TRY(dev_alloc(p->dev_mem, (void**)&s.near_v, 4 * (size_t)max_nnz_near));
            DRC_TRY(dev_alloc(p->dev_mem, (void**)&s.pins_rp, 4 * (size_t)(max_nets + 1)));
            DRC_TRY(dev_alloc(p->dev_mem, (void**)&s.pins_ci, 4 * (size_t)max_nnz_pins));
            DRC_TRY(dev_alloc(p->dev_mem, (void**)&s.pins_v, 4 * (size_t)max_nnz_pins));
            DRC_TRY(dev_alloc(p->dev_mem, (void**)&s.pinned_rp, 4 * (size_t)(max_cells + 1)));
            DRC_TRY(dev_alloc(p->dev_mem, (void**)&s.pinned_ci, 4 * (size_t)max_nnz_pins));
            DRC_TRY(dev_alloc(p->dev_mem, (void**)&s.pinned_v, 4 * (size_t)max_nnz_pins));
            DRC_TRY(dev_alloc(p->dev_mem, (void**)&s.X_cell, 4 * (size_t)max_cells * D));
            DRC_TRY(dev_alloc(p->dev_mem, (void**)&s.X_net, 4 * (size_t)max_nets * D));
            s.ws_t_bytes = dr_csr_transpose_workspace_bytes(max_nets, max_cells, max_nnz_pins);
            DRC_TRY(dev_alloc(p->dev_mem, &s.ws_t, s.ws_t_bytes));
            s.ws_n_bytes = dr_csr_normalize_workspace_bytes(DR_NORM_SYM, max_cells, max_nets > max_cells ? max_nets : max_cells, max_nnz_pins);
            DRC_TRY(dev_alloc(p->dev_mem, &s.ws_n, s.ws_n_bytes));
            s.off_near_ci = up256(4 * (size_t)(max_cells + 1));
            s.off_pins_rp = s.off_near_ci + up256(4 * (size_t)max_nnz_near);
            s.off_pins_ci = s.off_pins_rp + up256(4 * (size_t)(max_nets + 1));
            s.off_xc = s.off_pins_ci + up256(4 * (size_t)max_nnz_pins);
            s.off_xn = s.off_xc + up256(4 * (size_t)max_cells * D);
            s.stage_bytes = s.off_xn + up256(4 * (size_t)max_nets * D);
            void* h = nullptr;
            DRC_HIP(hipHostMalloc(&h, s.stage_bytes, hipHostMallocDefault));
            p->host_mem.push_back(h);
            s.stage = static_cast<char*>(h);
            DRC_TRY(heteroconv_create_capacity(&s.ctx, max_cells, max_nets, E, D, k_cell, k_cell, k_net, k_net, true));
            DRC_HIP(hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking));
            DRC_HIP(hipEventCreateWithFlags(&s.ready, hipEventDisableTiming));
            DRC_HIP(hipEventCreateWithFlags(&s.freed, hipEventDisableTiming));
        }
        DRC_HIP(hipDeviceSynchronize());
        return DR_OK;
    };
    const int rc = body();
    if (rc != DR_OK) {
        const std::string keep = dr_last_error();
        (void)dr_pipeline_destroy(p);
        return fail(rc, "%s", keep.c_str());
    }
    for (int t = 0; t < n_threads; ++t) p->workers.emplace_back(worker_main, p);
    *out = p;
    return DR_OK;
}

int dr_pipeline_submit(dr_pipeline* p, int32_t slot, const dr_host_graph* g) {
    DRC_REQUIRE(p != nullptr && g != nullptr, "dr_pipeline_submit: null argument");
    DRC_REQUIRE(slot >= 0 && slot < (int)p->slots.size(), "dr_pipeline_submit: slot %d out of range", slot);
    DRC_REQUIRE(g->n_cells >= 1 && g->n_nets >= 1 && g->nnz_near >= 0 && g->nnz_pins >= 0, "dr_pipeline_submit: bad graph sizes");
    DRC_REQUIRE(g->n_cells <= p->cap_cells && g->n_nets <= p->cap_nets && g->nnz_near <= p->cap_near && g->nnz_pins <= p->cap_pins,
                "dr_pipeline_submit: graph (%lld cells, %lld nets, %lld / %lld edges) exceeds the pipeline's capacity",
                (long long)g->n_cells, (long long)g->n_nets, (long long)g->nnz_near, (long long)g->nnz_pins);
    DRC_REQUIRE(g->near_rowptr && g->pins_rowptr && (g->nnz_near == 0 || g->near_colidx) && (g->nnz_pins == 0 || g->pins_colidx),
                "dr_pipeline_submit: null graph array");
    {
        std::lock_guard<std::mutex> lk(p->mu);
        Slot& s = p->slots[slot];
        DRC_REQUIRE(s.state == kIdle, "dr_pipeline_submit: slot %d is in use (acquire and release it first)", slot);
        s.job = *g;
        s.state = kQueued;
        p->queue.push_back(slot);
    }
    p->cv_job.notify_one();
    return DR_OK;
}

int dr_pipeline_acquire(dr_pipeline* p, int32_t slot, void* stream, dr_heteroconv** ctx, const float** X_cell,
                        const float** X_net) {
    DRC_REQUIRE(p != nullptr && ctx != nullptr, "dr_pipeline_acquire: null argument");
    DRC_REQUIRE(slot >= 0 && slot < (int)p->slots.size(), "dr_pipeline_acquire: slot %d out of range", slot);
    Slot& s = p->slots[slot];
    {
        std::unique_lock<std::mutex> lk(p->mu);
        DRC_REQUIRE(s.state != kIdle && s.state != kAcquired, "dr_pipeline_acquire: nothing was submitted to slot %d", slot);
        p->cv_done.wait(lk, [&] { return s.state == kReady || s.state == kFailed; });
        if (s.state == kFailed) {
            const int rc = s.rc;
            const std::string err = s.err;
            s.state = kIdle;
            return fail(rc, "dr_pipeline_acquire: slot %d: %s", slot, err.c_str());
        }
        s.state = kAcquired;
    }
    DRC_HIP(hipStreamWaitEvent(as_stream(stream), s.ready, 0));
    *ctx = s.ctx;
    if (X_cell) *X_cell = s.job.X_cell ? s.X_cell : nullptr;
    if (X_net) *X_net = s.job.X_net ? s.X_net : nullptr;
    return DR_OK;
}

int dr_pipeline_relations(dr_pipeline* p, int32_t slot, dr_csr* out) {
    DRC_REQUIRE(p != nullptr && out != nullptr, "dr_pipeline_relations: null argument");
    DRC_REQUIRE(slot >= 0 && slot < (int)p->slots.size(), "dr_pipeline_relations: slot %d out of range", slot);
    std::lock_guard<std::mutex> lk(p->mu);
    DRC_REQUIRE(p->slots[slot].state == kAcquired, "dr_pipeline_relations: slot %d is not acquired", slot);
    for (int i = 0; i < 3; ++i) out[i] = p->slots[slot].rel[i];
    return DR_OK;
}

int dr_pipeline_release(dr_pipeline* p, int32_t slot, void* stream) {
    DRC_REQUIRE(p != nullptr, "dr_pipeline_release: null pipeline");
    DRC_REQUIRE(slot >= 0 && slot < (int)p->slots.size(), "dr_pipeline_release: slot %d out of range", slot);
    Slot& s = p->slots[slot];
    {
        std::lock_guard<std::mutex> lk(p->mu);
        DRC_REQUIRE(s.state == kAcquired, "dr_pipeline_release: slot %d is not acquired", slot);
    }
    DRC_HIP(hipEventRecord(s.freed, as_stream(stream)));
    std::lock_guard<std::mutex> lk(p->mu);
    s.freed_pending = true;
    s.state = kIdle;
    return DR_OK;
}

}  // extern "C"
