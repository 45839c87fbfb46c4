#!/usr/bin/env python3
"""Benchmark of the HeteroConv DR-SpMM hot path on one MI355X.

A *step* (what `value`, `ms_per_step`, `steps` and `warmup` refer to) is one pass of the D-ReLU / DR-SpMM kernels of
a HeteroConv layer, forward and backward, over one seeded synthetic circuit graph: `dr_topk` of both node types,
`dr_spmm_fwd` of the three relations and `dr_spmm_bwd` of the three transposed relations -- eight launches through
the C ABI, forked from the caller's stream onto three streams (one per relation, paper Section 3.4) and joined by
events, with no host wait in between.  `value` = the compulsory bytes of those eight kernels (every array once)
divided by the time of that region.  Graph setup (edge values, transposes) is done once before the timed region;
every input is resident in HBM when it starts.

Reported beside it on the same JSON line: `dr_kernels` (each of the eight kernels alone on its stream, HIP events
around every launch), `roofline` (the longest of them against the HBM roof), `layer_step` (the whole layer,
heteroconv_fwd + heteroconv_bwd with projections, merge and weight gradients), `k_sweep` (the region at k = 8, 16, 32,
64 on the `large` workload) and `cpu_baseline` (the oracle's functions for the same eight operations on the same
inputs, one host thread).  `operation_models()` / `kernel_models()` below are the byte models.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix, published


# ----------------------------------------------------------------------------------------------------
# algorithmic (compulsory) bytes and flops per kernel: every array the kernel must read or write, once
# ----------------------------------------------------------------------------------------------------

def operation_models(Nc, Nn, E, D, ks):
    """{operation name: (bytes, flops)} for one step: the step's work as a fixed list of operations, which is what
    `value` counts (fusing two of them into one kernel later does not change the numerator).  E = dict(near=,
    pins=, pinned=); ks = (k_near, k_pins, k_self, k_pinned): D-ReLU widths of the cells for near / for pins and
    of the nets for the pins self term / for pinned (k_cell, k_cell, k_net, k_net with one K per node type)."""
    k_near, k_pins, k_self, k_pinned = ks
    W = 4 * D * D

    def topk(n, k):
        return 4 * n * D + 6 * n * k, n * D

    def fwd(M, N, e, k):      # rowptr + (colidx, vals) + CBSR of the sources + dense output
        return 4 * (M + 1) + 8 * e + 6 * N * k + 4 * M * D, 2 * e * k

    def bwd(Nsrc, M, e, k):   # rowptr + (colidx, vals) + saved idx + gathered dH + compact output
        return 4 * (Nsrc + 1) + 8 * e + 2 * Nsrc * k + min(4 * e * k, 4 * M * D) + 4 * Nsrc * k, 2 * e * k

    m = {}
    # a node type read at two widths is selected at both in one pass over its embeddings
    m["dr_topk.cell"] = topk(Nc, k_near + (k_pins if k_pins != k_near else 0))
    m["dr_topk.net"] = topk(Nn, k_pinned + (k_self if k_self != k_pinned else 0))
    m["dr_spmm_fwd.near"] = fwd(Nc, Nc, E["near"], k_near)
    m["dr_spmm_fwd.pins"] = fwd(Nn, Nc, E["pins"], k_pins)
    m["dr_spmm_fwd.pinned"] = fwd(Nc, Nn, E["pinned"], k_pinned)
    m["proj.near"] = (6 * Nc * k_near + 4 * Nc * D + 2 * W + 4 * Nc * D, 2 * Nc * D * (D + D))
    m["proj.pins"] = (6 * Nn * k_self + 4 * Nn * D + 2 * W + 4 * Nn * D, 2 * Nn * D * (D + D))
    m["proj.pinned+merge"] = (4 * Nc * D + W + 8 * Nc * D + Nc * D, 2 * Nc * D * D)
    m["dproj.near"] = (5 * Nc * D + W + 4 * Nc * D, 2 * Nc * D * D)
    m["dproj.pins"] = (4 * Nn * D + W + 4 * Nn * D, 2 * Nn * D * D)
    m["dproj.pinned"] = (5 * Nc * D + W + 4 * Nc * D, 2 * Nc * D * D)
    m["dr_spmm_bwd.near"] = bwd(Nc, Nc, E["near"], k_near)
    m["dr_spmm_bwd.pins"] = bwd(Nc, Nn, E["pins"], k_pins)
    m["dr_spmm_bwd.pinned"] = bwd(Nn, Nc, E["pinned"], k_pinned)
    # self-term gradient sampled at the saved indices, added to the compact SpMM gradient(s), written as dense dX
    cell_sets = 6 * Nc * k_near + (6 * Nc * k_pins if k_pins != k_near else 0)
    net_sets = 6 * Nn * k_pinned + (2 * Nn * k_self if k_self != k_pinned else 0)
    m["dself.near+dX"] = (5 * Nc * D + W + cell_sets + 4 * Nc * D, 2 * Nc * D * D)
    m["dself.pins+dX"] = (4 * Nn * D + W + net_sets + 4 * Nn * D, 2 * Nn * D * D)
    m["wgrad.neigh_near"] = (4 * Nc * D + 5 * Nc * D + W, 2 * Nc * D * D)
    m["wgrad.self_near"] = (6 * Nc * k_near + 5 * Nc * D + W, 2 * Nc * D * D)
    m["wgrad.neigh_pins"] = (8 * Nn * D + W, 2 * Nn * D * D)
    m["wgrad.self_pins"] = (6 * Nn * k_self + 4 * Nn * D + W, 2 * Nn * D * D)
    m["wgrad.pinned"] = (4 * Nc * D + 5 * Nc * D + W, 2 * Nc * D * D)
    return m


def kernel_models(Nc, Nn, E, D, ks):
    """{kernel name: (bytes, flops)} for the kernels as launched (the names heteroconv_kernel_times reports): the
    operations above, except that the two weight gradients of a SageConv module are one kernel that reads the
    shared upstream gradient once."""
    k_near, k_pins, k_self, k_pinned = ks
    W = 4 * D * D
    m = operation_models(Nc, Nn, E, D, ks)
    for n in ("wgrad.neigh_near", "wgrad.self_near", "wgrad.neigh_pins", "wgrad.self_pins"):
        del m[n]
    m["wgrad.near"] = (4 * Nc * D + 6 * Nc * k_near + 5 * Nc * D + 2 * W, 4 * Nc * D * D)
    m["wgrad.pins"] = (4 * Nn * D + 6 * Nn * k_self + 4 * Nn * D + 2 * W, 4 * Nn * D * D)
    return m


DR_KERNELS = ("dr_topk.cell", "dr_topk.net", "dr_spmm_fwd.near", "dr_spmm_fwd.pins", "dr_spmm_fwd.pinned",
              "dr_spmm_bwd.near", "dr_spmm_bwd.pins", "dr_spmm_bwd.pinned")


REL_TYPES = dict(near=("cell", "cell"), pins=("cell", "net"), pinned=("net", "cell"))   # relation -> (source, destination) type


class DrRegion:
    """Buffers and launch sequence of the eight D-ReLU / DR-SpMM kernels of one layer pass.  The backward kernels read
    seeded N(0,1) upstream gradients of the destination type (in the layer they come from the projection gradients,
    which are not part of this region) and write one compact gradient each."""

    def __init__(self, P, torch, rel, rel_t, X, dH, D, k, near_plan=None):
        self.P, self.torch, self.rel, self.rel_t, self.X, self.dH, self.D, self.k = P, torch, rel, rel_t, X, dH, D, k
        self.near_plan = near_plan      # dr_spmm_plan of the transposed `near` relation in placement order, or None
        f32, i16 = torch.float32, torch.int16
        n = dict(cell=X["cell"].shape[0], net=X["net"].shape[0])
        self.vals = {t: torch.empty((n[t], k), dtype=f32, device="cuda") for t in n}
        self.idx = {t: torch.empty((n[t], k), dtype=i16, device="cuda") for t in n}
        self.H = {r: torch.empty((n[REL_TYPES[r][1]], D), dtype=f32, device="cuda") for r in REL_TYPES}
        self.G = {r: torch.empty((n[REL_TYPES[r][0]], k), dtype=f32, device="cuda") for r in REL_TYPES}
        self.side = (torch.cuda.Stream(), torch.cuda.Stream())          # default priority
        self.ev = {n_: torch.cuda.Event() for n_ in ("fork", "cell", "pins", "pinned")}

    def kernels(self):
        """{name: callable(stream)} -- one launch each through the C ABI."""
        P, D, k = self.P, self.D, self.k
        out = {}
        for t in ("cell", "net"):
            out[f"dr_topk.{t}"] = (lambda s, t=t: P.dr_topk(self.X[t], k, self.vals[t], self.idx[t], stream=s))
        for r, (src, dst) in REL_TYPES.items():
            out[f"dr_spmm_fwd.{r}"] = (lambda s, r=r, src=src: P.dr_spmm_fwd(self.rel[r], self.vals[src], self.idx[src], D, k,
                                                                               self.H[r], stream=s))
            if r == "near" and self.near_plan is not None:
                out["dr_spmm_bwd.near"] = (lambda s: self.near_plan.dr_spmm_bwd_planned(self.dH["cell"], self.idx["cell"], k,
                                                                                          self.G["near"], stream=s))
            else:
                out[f"dr_spmm_bwd.{r}"] = (lambda s, r=r, src=src, dst=dst: P.dr_spmm_bwd(self.rel_t[r], self.dH[dst], self.idx[src],
                                                                                           D, k, self.G[r], stream=s))
        return out

    def run(self, concurrent=True):
        """One pass.  concurrent: near on the caller's stream, pins and pinned on two side streams; pins waits for the
        cells' D-ReLU.  Otherwise all eight launches on the caller's stream."""
        K = self.kernels()
        main = self.torch.cuda.current_stream()
        if not concurrent:
            for n_ in ("dr_topk.cell", "dr_spmm_fwd.near", "dr_spmm_bwd.near", "dr_spmm_fwd.pins", "dr_spmm_bwd.pins",
                       "dr_topk.net", "dr_spmm_fwd.pinned", "dr_spmm_bwd.pinned"):
                K[n_](main)
            return
        s_pins, s_pinned = self.side
        ev = self.ev
        ev["fork"].record(main)
        s_pins.wait_event(ev["fork"])
        s_pinned.wait_event(ev["fork"])
        K["dr_topk.cell"](main)
        ev["cell"].record(main)
        K["dr_topk.net"](s_pinned)
        s_pins.wait_event(ev["cell"])
        K["dr_spmm_fwd.pins"](s_pins)
        K["dr_spmm_fwd.near"](main)
        K["dr_spmm_fwd.pinned"](s_pinned)
        K["dr_spmm_bwd.pins"](s_pins)
        K["dr_spmm_bwd.near"](main)
        K["dr_spmm_bwd.pinned"](s_pinned)
        ev["pins"].record(s_pins)
        ev["pinned"].record(s_pinned)
        main.wait_event(ev["pins"])
        main.wait_event(ev["pinned"])

    def time_region(self, warmup, steps, concurrent=True):
        """(wall ms per pass between device synchronisations, HIP-event ms per pass on the caller's stream)."""
        torch = self.torch
        for _ in range(warmup):
            self.run(concurrent)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        a.record()
        for _ in range(steps):
            self.run(concurrent)
        b.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        return wall, a.elapsed_time(b) / steps

    def time_kernels(self, warmup, iters):
        """Each kernel alone on the caller's stream: HIP events around every launch; {name: (mean, median, min) ms}."""
        torch = self.torch
        main = torch.cuda.current_stream()
        self.run(False)                                     # every buffer a kernel reads holds valid contents
        out = {}
        for name, launch in self.kernels().items():
            for _ in range(warmup):
                launch(main)
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
            for a, b in evs:
                a.record(main)
                launch(main)
                b.record(main)
            torch.cuda.synchronize()
            ms = sorted(a.elapsed_time(b) for a, b in evs)
            out[name] = (sum(ms) / len(ms), ms[len(ms) // 2], ms[0])
        return out


def dr_models(Nc, Nn, E, D, k):
    m = operation_models(Nc, Nn, E, D, (k, k, k, k))
    return {n: m[n] for n in DR_KERNELS}


def cpu_baseline_dr(g, T, D, k):
    """The oracle's functions for the eight operations of the timed region -- orc_topk x2, orc_spmm_fwd x3,
    orc_spmm_bwd x3 -- on the benchmark's own graph and tensors, one after the other on one host thread."""
    import numpy as np
    import oracle
    rel = dict(near=oracle.relation(g.near, oracle.NORM_MEAN), pins=oracle.relation(g.pins, oracle.NORM_MEAN),
               pinned=oracle.relation(g.pinned, oracle.NORM_SYM))
    tr = {n: oracle.csr_transpose(rel[n].M, rel[n].N, rel[n].rowptr, rel[n].colidx, rel[n].vals) for n in rel}   # setup, not timed
    X = dict(cell=T.X_cell, net=T.X_net)
    dH = dict(cell=T.dY_cell, net=T.dY_net)
    secs, cb = {}, {}
    for t in ("cell", "net"):
        t0 = time.perf_counter()
        cb[t] = oracle.topk(X[t], k)
        secs[f"dr_topk.{t}"] = time.perf_counter() - t0
    for r, (src, dst) in REL_TYPES.items():
        t0 = time.perf_counter()
        oracle.spmm_fwd(rel[r].rowptr, rel[r].colidx, rel[r].vals, cb[src][0], cb[src][1], D)
        secs[f"dr_spmm_fwd.{r}"] = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.spmm_bwd(*tr[r], dH[dst], cb[src][1])
        secs[f"dr_spmm_bwd.{r}"] = time.perf_counter() - t0
    return secs


def cpu_baseline_layer(name: str, D: int, ks, scale: int):
    """The oracle's layer forward + backward on a 1/scale-size graph drawn from the same laws."""
    import oracle
    from oracle import per_relation as opr
    from circuit_synth import make_graph, make_tensors, workload
    w = workload(name)
    gw, gh = w["grid"]
    f = scale ** 0.5
    Nc, Nn = w["Nc"] // scale, w["Nn"] // scale
    grid = (max(8, int(round(gw / f))), max(8, int(round(gh / f))))
    while grid[0] * grid[1] < Nc:
        grid = (grid[0] + 1, grid[1])
    g = make_graph(name, seed=0, Nc=Nc, Nn=Nn, grid=grid)
    T = make_tensors(Nc, Nn, D, seed=0)
    rels = (oracle.relation(g.near, oracle.NORM_MEAN), oracle.relation(g.pins, oracle.NORM_MEAN),
            oracle.relation(g.pinned, oracle.NORM_SYM))
    one_k = ks[0] == ks[1] and ks[2] == ks[3]
    t0 = time.perf_counter()
    if one_k:
        of = oracle.heteroconv_fwd(*rels, T.X_cell, T.X_net, T.W, ks[0], ks[3])
        oracle.heteroconv_bwd(*rels, T.W, of, T.dY_cell, T.dY_net)
    else:
        of = opr.heteroconv_fwd(*rels, T.X_cell, T.X_net, T.W, opr.Ks(*ks))
        opr.heteroconv_bwd(*rels, T.W, of, T.dY_cell, T.dY_net)
    dt = time.perf_counter() - t0
    models = operation_models(Nc, Nn, dict(near=g.near.nnz, pins=g.pins.nnz, pinned=g.pinned.nnz), D, ks)
    step_bytes = sum(b for b, _ in models.values())
    return dict(value=round(step_bytes / dt / 1e9, 4), unit="GB/s", seconds=round(dt, 3),
                sample=f"oracle HeteroConv layer fwd+bwd (fp64, 1 thread) on a 1/{scale}-scale '{name}' graph: {Nc} cells, "
                       f"{Nn} nets, E_near={g.near.nnz}, E_pins={g.pins.nnz}, D={D}; {step_bytes / 1e6:.1f} MB of the layer's "
                       f"algorithmic bytes")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="large", help="tiny | small | medium | large | subgraph")
    ap.add_argument("--k", type=int, default=None, help="D-ReLU k of the headline (default: the workload's)")
    ap.add_argument("--only", choices=("all", "dr", "layer"), default="all",
                    help="dr: only the timed D-ReLU / DR-SpMM region; layer: only the whole-layer steps (for profiler runs)")
    ap.add_argument("--serial", action="store_true", help="the region's eight launches on one stream (for counter runs)")
    ap.add_argument("--no-k-sweep", action="store_true")
    ap.add_argument("--no-staging", action="store_true",
                    help="transposed `near` DR-SpMM without the LDS-staged tiles (the plain gather kernel, as for pins / pinned)")
    ap.add_argument("--kernel-iters", type=int, default=50, help="launches per kernel in the per-kernel timing pass")
    ap.add_argument("--layer-steps", type=int, default=20)
    ap.add_argument("--k-per-relation", default=None,
                    help="layer step with one K per edge type: 'k_near,k_pins,k_pinned', or 'best' = what --profile-k picks")
    ap.add_argument("--profile-k", action="store_true",
                    help="optimal-K profiling of the workload's graph over K = 2..64 (reported as k_profile)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-scale", type=int, default=None, help="oracle layer sample = 1/scale of the workload")
    ap.add_argument("--no-profile-events", action="store_true", help="layer steps without per-kernel HIP events")
    ap.add_argument("--overlap", choices=("auto", "on", "off"), default="auto",
                    help="layer step: three streams (on), one stream (off), or the library's size rule")
    ap.add_argument("--permute-cells", action="store_true",
                    help="sensitivity run: relabel the cells at random (removes the grid locality of `near`)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy a few times (known traffic, for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path is single-GPU; sharding it over several GPUs is "
              "a design note, not code); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2508_16769_amd as P
    from circuit_synth import make_graph, make_tensors, workload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.copy_calibration:
        a = torch.ones(256 * 1024 * 1024, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 5
        print(json.dumps({"copy_bytes_read": a.numel() * 4, "copy_bytes_written": a.numel() * 4,
                          "ms": round(dt * 1e3, 4), "GBs": round(2 * a.numel() * 4 / dt / 1e9, 1)}), flush=True)
        return 0
    w = workload(args.workload)
    D = w["D"]
    k = args.k if args.k is not None else w["k"]

    t_setup = time.perf_counter()
    g = make_graph(args.workload, seed=0)
    if args.permute_cells:
        from circuit_synth.generate import permute_cells
        g = permute_cells(g, seed=0)
    T = make_tensors(g.Nc, g.Nn, D, seed=0)
    E = dict(near=g.near.nnz, pins=g.pins.nnz, pinned=g.pinned.nnz)

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    rel = dict(near=P.device_relation(g.near, P.DR_NORM_MEAN), pins=P.device_relation(g.pins, P.DR_NORM_MEAN),
               pinned=P.device_relation(g.pinned, P.DR_NORM_SYM))
    torch.cuda.synchronize()
    t_graph = time.perf_counter()
    rel_t = {r: P.device_transpose(rel[r]) for r in rel}
    torch.cuda.synchronize()
    t_transposes = time.perf_counter() - t_graph
    X = dict(cell=dev(T.X_cell), net=dev(T.X_net))
    dY = dict(cell=dev(T.dY_cell), net=dev(T.dY_net))
    near_plan, plan_note = None, "off"
    if not args.no_staging and g.cell_order is not None:
        t_plan = time.perf_counter()
        try:
            near_plan = P.SpmmPlan(rel_t["near"], D, dev(g.cell_order))
            n_tiles, reuse = near_plan.dr_spmm_plan_info()
            plan_note = (f"near^T in placement order: {n_tiles} tiles, {reuse:.2f} edges per staged dH row, "
                         f"plan built in {time.perf_counter() - t_plan:.2f} s")
        except P.DrError as e:
            if e.code != P.DR_ERR_UNSUPPORTED:
                raise
            plan_note = f"refused: {e}"
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup
    workload_label = (f"{args.workload}: {g.Nc} cells, {g.Nn} nets, E_near={E['near']}, E_pins={E['pins']}, D={D}, k={k}"
                      + (" (cell ids randomly permuted)" if args.permute_cells else ""))

    out = {
        "metric": "HeteroConv DR-SpMM fwd+bwd effective GB/s",
        "value": None, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": None,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload_label,
                   "timed_region": "dr_topk x2 + dr_spmm_fwd x3 + dr_spmm_bwd x3, " +
                                   ("one stream" if args.serial else "three streams (one per relation), joined by events"),
                   "lds_staging": plan_note, "setup_s": round(t_setup, 2), "transposes_s": round(t_transposes, 3)},
    }

    # ------------------------------------------------------------------------------------------------
    # the timed region: the eight D-ReLU / DR-SpMM kernels, forked on three streams
    # ------------------------------------------------------------------------------------------------
    if args.only in ("all", "dr"):
        region = DrRegion(P, torch, rel, rel_t, X, dY, D, k, near_plan)
        models = dr_models(g.Nc, g.Nn, E, D, k)
        dr_bytes = sum(b for b, _ in models.values())
        dr_flops = sum(f for n, (_, f) in models.items() if n.startswith("dr_spmm"))
        wall_ms, event_ms = region.time_region(args.warmup, args.steps, concurrent=not args.serial)
        out["value"] = round(dr_bytes / (wall_ms * 1e-3) / 1e9, 1)
        out["ms_per_step"] = round(wall_ms, 4)
        out["config"].update(step_algorithmic_MB=round(dr_bytes / 1e6, 1), frac_of_hbm_peak=round(out["value"] / HBM_PEAK_GBS, 4),
                             region_event_ms=round(event_ms, 4), GFLOPs=round(dr_flops / (wall_ms * 1e-3) / 1e9, 1))
        if args.only == "all":
            per = region.time_kernels(10, max(10, args.kernel_iters))
            kernels = {n: dict(ms=round(avg, 4), ms_median=round(med, 4), ms_min=round(mn, 4), MB=round(models[n][0] / 1e6, 2),
                               GBs=round(models[n][0] / (avg * 1e-3) / 1e9, 1), GFLOPs=round(models[n][1] / (avg * 1e-3) / 1e9, 1))
                       for n, (avg, med, mn) in per.items()}
            total = sum(v["ms"] for v in kernels.values())
            out["dr_kernels"] = dict(protocol=f"each kernel alone on its stream, 10 warm-ups + {max(10, args.kernel_iters)} launches, "
                                              "HIP events around every launch", sum_ms=round(total, 4),
                                     GBs_serialized=round(dr_bytes / (total * 1e-3) / 1e9, 1), kernels=kernels)
            dom = max(kernels, key=lambda n: kernels[n]["ms"])
            b, f = models[dom]
            ach = b / (kernels[dom]["ms"] * 1e-3) / 1e9
            traffic, source = None, None
            tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
            if os.path.exists(tpath) and not args.permute_cells:
                try:
                    tab = json.load(open(tpath))
                    traffic = tab.get(f"{args.workload}.k{k}", {}).get(dom)
                    source = tab.get("measured", {}).get(f"{args.workload}.k{k}")
                except Exception:
                    traffic = None
            out["roofline"] = dict(bound="hbm", achieved=round(ach, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                                   frac=round(ach / HBM_PEAK_GBS, 4), traffic=traffic, kernel=dom, avg_ms=kernels[dom]["ms"],
                                   algorithmic_bytes=b)
            if traffic:
                out["roofline"]["traffic_source"] = source or "profiles/hbm_traffic.json (rocprofv3 FETCH_SIZE x 2.0 + WRITE_SIZE)"
                out["roofline"]["measured_hbm_GBs"] = round(traffic / (kernels[dom]["ms"] * 1e-3) / 1e9, 1)
            # the same region on one stream, for the value of relation concurrency
            s_wall, _ = region.time_region(3, max(5, args.steps // 2), concurrent=args.serial)
            out["config"]["region_ms_other_schedule"] = {("three streams" if args.serial else "one stream"): round(s_wall, 4)}
        del region

        if args.only == "all" and args.workload == "large" and not args.no_k_sweep:
            sweep = {}
            for kk in (8, 16, 32, 64):
                rg = DrRegion(P, torch, rel, rel_t, X, dY, D, kk, near_plan)
                m = dr_models(g.Nc, g.Nn, E, D, kk)
                bb = sum(b for b, _ in m.values())
                ff = sum(f for n, (_, f) in m.items() if n.startswith("dr_spmm"))
                wms, _ = rg.time_region(5, 20, concurrent=not args.serial)
                sweep[f"k{kk}"] = dict(ms=round(wms, 4), MB=round(bb / 1e6, 1), GBs=round(bb / (wms * 1e-3) / 1e9, 1),
                                       frac_of_hbm_peak=round(bb / (wms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                       GFLOPs=round(ff / (wms * 1e-3) / 1e9, 1))
                del rg
            out["k_sweep"] = sweep

    # ------------------------------------------------------------------------------------------------
    # the whole layer: heteroconv_fwd + heteroconv_bwd (projections, merge, weight gradients included)
    # ------------------------------------------------------------------------------------------------
    ks = (k, k, k, k)
    if args.only in ("all", "layer"):
        layer = P.HeteroConv(rel["near"], rel["pins"], rel["pinned"], D, k, k)
        k_profile = None
        if args.profile_k or args.k_per_relation == "best":
            cand = [c for c in (2, 4, 8, 16, 32, 64) if c <= D]
            tp = time.perf_counter()
            ms_f, ms_b, best = layer.heteroconv_profile_k(X["cell"], X["net"], cand, warmup=2, reps=5)
            k_profile = dict(candidates=cand, relations=["near", "pins", "pinned"],
                             ms_fwd=[[round(v, 4) for v in r] for r in ms_f], ms_bwd=[[round(v, 4) for v in r] for r in ms_b],
                             best=list(best), seconds=round(time.perf_counter() - tp, 3))
            out["k_profile"] = k_profile
        if args.k_per_relation:
            kk = k_profile["best"] if args.k_per_relation == "best" else [int(v) for v in args.k_per_relation.split(",")]
            if len(kk) != 3:
                print("bench.py: --k-per-relation takes k_near,k_pins,k_pinned", file=sys.stderr)
                return 2
            layer.heteroconv_destroy()
            layer = P.HeteroConv(rel["near"], rel["pins"], rel["pinned"], D, per_relation=kk)
        ks = layer.heteroconv_get_k()
        layer_staged = False
        if not args.no_staging and g.cell_order is not None:
            layer_staged = layer.heteroconv_set_cell_order(dev(g.cell_order))
        layer.heteroconv_set_overlap({"auto": P.DR_OVERLAP_AUTO, "on": P.DR_OVERLAP_ON, "off": P.DR_OVERLAP_OFF}[args.overlap])
        saved = layer.alloc_saved()
        Wd = {n: dev(T.W[n]) for n in P.WEIGHT_NAMES}
        Y_cell = torch.empty((g.Nc, D), dtype=torch.float32, device="cuda")
        Y_net = torch.empty((g.Nn, D), dtype=torch.float32, device="cuda")
        dX_cell, dX_net = torch.empty_like(Y_cell), torch.empty_like(Y_net)
        dW = {n: torch.empty((D, D), dtype=torch.float32, device="cuda") for n in P.WEIGHT_NAMES}

        def step():
            layer.heteroconv_fwd(X["cell"], X["net"], Wd, Y_cell, Y_net, saved)
            layer.heteroconv_bwd(dY["cell"], dY["net"], Wd, saved, dX_cell, dX_net, dW)

        n_steps = args.steps if args.only == "layer" else args.layer_steps
        n_warm = args.warmup if args.only == "layer" else 3
        for _ in range(n_warm):
            step()
        torch.cuda.synchronize()
        if not args.no_profile_events:
            layer.heteroconv_profile(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_steps):
            step()
        torch.cuda.synchronize()
        layer_ms = (time.perf_counter() - t0) * 1e3 / n_steps
        times = {} if args.no_profile_events else layer.heteroconv_kernel_times()
        layer.heteroconv_profile(False)
        lmodels = kernel_models(g.Nc, g.Nn, E, D, ks)
        step_bytes = sum(b for b, _ in operation_models(g.Nc, g.Nn, E, D, ks).values())
        lk = {}
        for name, (ms_sum, cnt) in times.items():
            if cnt:
                avg = ms_sum / cnt
                b, f = lmodels[name]
                lk[name] = dict(ms=round(avg, 4), GBs=round(b / (avg * 1e-3) / 1e9, 1), GFLOPs=round(f / (avg * 1e-3) / 1e9, 1),
                                MB=round(b / 1e6, 2))
        klabel = str(k) if not args.k_per_relation else "k_near/k_pins/k_pinned=" + "/".join(str(v) for v in (ks[0], ks[1], ks[3]))
        out["layer_step"] = dict(what=f"heteroconv_fwd + heteroconv_bwd, k={klabel}, relation_overlap={args.overlap}, "
                                      f"near^T on LDS-staged tiles: {'yes' if layer_staged else 'no'}, "
                                      f"{n_warm} warm-ups + {n_steps} steps, per-kernel HIP events "
                                      + ("off" if args.no_profile_events else "on"),
                                 ms_per_step=round(layer_ms, 4), algorithmic_MB=round(step_bytes / 1e6, 1),
                                 GBs=round(step_bytes / (layer_ms * 1e-3) / 1e9, 1), kernels=lk)
        if args.only == "layer":
            out["value"] = out["layer_step"]["GBs"]
            out["ms_per_step"] = out["layer_step"]["ms_per_step"]
            out["metric"] = "HeteroConv layer fwd+bwd effective GB/s (all operations)"
        layer.heteroconv_destroy()

    if not args.no_cpu_baseline:
        secs = cpu_baseline_dr(g, T, D, k)
        total = sum(secs.values())
        dr_bytes = sum(b for b, _ in dr_models(g.Nc, g.Nn, E, D, k).values())
        scale = args.cpu_scale or max(1, g.Nc // 200000)
        out["cpu_baseline"] = dict(
            value=round(dr_bytes / total / 1e9, 4), unit="GB/s", cores=1, kind="oracle",
            sample=f"the whole workload ({workload_label}): orc_topk x2, orc_spmm_fwd x3, orc_spmm_bwd x3 on the benchmark's own "
                   f"graph and tensors (fp64, one thread, one call after the other); {total:.1f} s for the same "
                   f"{dr_bytes / 1e6:.1f} MB of compulsory bytes the GPU region is credited with",
            seconds=round(total, 3), seconds_per_function={n: round(v, 3) for n, v in secs.items()},
            host_cores_available=len(os.sched_getaffinity(0)),
            layer=cpu_baseline_layer(args.workload, D, ks, scale))
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
