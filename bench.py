#!/usr/bin/env python3
"""Benchmark of the HeteroConv DR-SpMM hot path on one MI355X.

A *step* is one HeteroConv forward + backward over one seeded synthetic circuit graph: D-ReLU top-k of
both node types, the three DR-SpMM forwards, the projections and max-merge, and the whole backward
(projection gradients, the three transposed DR-SpMMs gated by the saved indices, weight gradients).
Graph setup (edge values, transposes) is done once before the timed region.  Inputs are resident in HBM
when the timed region starts.

Prints ONE JSON line; `operation_models()` / `kernel_models()` below are the byte models behind `value` and `roofline`.
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


def cpu_baseline(name: str, D: int, ks, scale: int):
    """The oracle's layer forward + backward on a 1/scale-size graph drawn from the same laws."""
    import numpy as np  # noqa: F401
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
    return dict(value=round(step_bytes / dt / 1e9, 4), unit="GB/s", cores=1, kind="oracle",
                sample=f"oracle HeteroConv fwd+bwd (fp64, 1 thread) on a 1/{scale}-scale '{name}' graph: "
                       f"{Nc} cells, {Nn} nets, E_near={g.near.nnz}, E_pins={g.pins.nnz}, D={D}, "
                       f"k={ks[0] if one_k and ks[0] == ks[3] else '/'.join(map(str, ks))}; "
                       f"{dt:.2f} s for {step_bytes / 1e6:.1f} MB of algorithmic traffic",
                seconds=round(dt, 3), host_cores_available=len(os.sched_getaffinity(0)))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large", help="tiny | small | medium | large | subgraph")
    ap.add_argument("--k", type=int, default=None, help="D-ReLU k (default: the workload's; large sweeps 8..64)")
    ap.add_argument("--k-per-relation", default=None,
                    help="one K per edge type: 'k_near,k_pins,k_pinned', or 'best' = what --profile-k picks")
    ap.add_argument("--profile-k", action="store_true",
                    help="optimal-K profiling of the workload's graph over K = 2..64 before the timed steps "
                         "(reported as k_profile)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-scale", type=int, default=None, help="oracle sample = 1/scale of the workload")
    ap.add_argument("--no-profile-events", action="store_true", help="do not bracket kernels with HIP events")
    ap.add_argument("--overlap", choices=("auto", "on", "off"), default="auto",
                    help="relation concurrency: three streams (on), one stream (off), or the library's size rule")
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

    near = P.device_relation(g.near, P.DR_NORM_MEAN)
    pins = P.device_relation(g.pins, P.DR_NORM_MEAN)
    pinned = P.device_relation(g.pinned, P.DR_NORM_SYM)
    torch.cuda.synchronize()
    t_graph = time.perf_counter()
    layer = P.HeteroConv(near, pins, pinned, D, k, k)     # device transposes + scratch
    t_ctx = time.perf_counter() - t_graph
    X_cell, X_net = dev(T.X_cell), dev(T.X_net)
    k_profile = None
    if args.profile_k or args.k_per_relation == "best":
        cand = [c for c in (2, 4, 8, 16, 32, 64) if c <= D]
        tp = time.perf_counter()
        ms_f, ms_b, best = layer.heteroconv_profile_k(X_cell, X_net, cand, warmup=2, reps=5)
        k_profile = dict(candidates=cand, relations=["near", "pins", "pinned"],
                         ms_fwd=[[round(v, 4) for v in r] for r in ms_f], ms_bwd=[[round(v, 4) for v in r] for r in ms_b],
                         best=list(best), seconds=round(time.perf_counter() - tp, 3))
    if args.k_per_relation:
        kk = k_profile["best"] if args.k_per_relation == "best" else [int(v) for v in args.k_per_relation.split(",")]
        if len(kk) != 3:
            print("bench.py: --k-per-relation takes k_near,k_pins,k_pinned", file=sys.stderr)
            return 2
        layer.heteroconv_destroy()
        layer = P.HeteroConv(near, pins, pinned, D, per_relation=kk)
    ks = layer.heteroconv_get_k()
    klabel = str(k) if not args.k_per_relation else "k_near/k_pins/k_pinned=" + "/".join(str(v) for v in (ks[0], ks[1], ks[3]))
    layer.heteroconv_set_overlap({"auto": P.DR_OVERLAP_AUTO, "on": P.DR_OVERLAP_ON, "off": P.DR_OVERLAP_OFF}[args.overlap])
    saved = layer.alloc_saved()
    Wd = {n: dev(T.W[n]) for n in P.WEIGHT_NAMES}
    dY_cell, dY_net = dev(T.dY_cell), dev(T.dY_net)
    Y_cell = torch.empty((g.Nc, D), dtype=torch.float32, device="cuda")
    Y_net = torch.empty((g.Nn, D), dtype=torch.float32, device="cuda")
    dX_cell, dX_net = torch.empty_like(Y_cell), torch.empty_like(Y_net)
    dW = {n: torch.empty((D, D), dtype=torch.float32, device="cuda") for n in P.WEIGHT_NAMES}
    del T
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup

    def step():
        layer.heteroconv_fwd(X_cell, X_net, Wd, Y_cell, Y_net, saved)
        layer.heteroconv_bwd(dY_cell, dY_net, Wd, saved, dX_cell, dX_net, dW)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if not args.no_profile_events:
        layer.heteroconv_profile(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    times = {} if args.no_profile_events else layer.heteroconv_kernel_times()
    layer.heteroconv_profile(False)

    models = kernel_models(g.Nc, g.Nn, E, D, ks)
    step_bytes = sum(b for b, _ in operation_models(g.Nc, g.Nn, E, D, ks).values())
    dr_bytes = sum(models[n][0] for n in DR_KERNELS if n in models)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    kernels = {}
    for name, (ms_sum, cnt) in times.items():
        if cnt == 0:
            continue
        avg = ms_sum / cnt
        b, f = models[name]
        kernels[name] = dict(ms=round(avg, 4), GBs=round(b / (avg * 1e-3) / 1e9, 1),
                             GFLOPs=round(f / (avg * 1e-3) / 1e9, 1), MB=round(b / 1e6, 2))
    roofline = None
    dr_region = None
    if kernels:
        # dominant kernel: the kernel symbol with the largest share of the step (launches of one instantiation are
        # named family.relation), represented by its longest launch
        fam = {}
        for n in kernels:
            fam[n.split(".")[0]] = fam.get(n.split(".")[0], 0.0) + kernels[n]["ms"]
        top = max(fam, key=fam.get)
        dom = max((n for n in kernels if n.split(".")[0] == top), key=lambda n: kernels[n]["ms"])
        b, f = models[dom]
        avg_s = kernels[dom]["ms"] * 1e-3
        traffic = None
        tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
        if os.path.exists(tpath):
            try:
                tkey = f"{args.workload}.k{k}" if not args.k_per_relation else None
                traffic = json.load(open(tpath)).get(tkey, {}).get(dom)
            except Exception:
                traffic = None
        intensity = f / b
        if intensity > MFMA_FP32_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
            ach = f / avg_s / 1e12
            roofline = dict(bound="mfma", achieved=round(ach, 2), peak=MFMA_FP32_PEAK_TFLOPS, unit="TFLOP/s",
                            frac=round(ach / MFMA_FP32_PEAK_TFLOPS, 4), traffic=traffic, kernel=dom,
                            avg_ms=kernels[dom]["ms"])
        else:
            ach = b / avg_s / 1e9
            roofline = dict(bound="hbm", achieved=round(ach, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                            frac=round(ach / HBM_PEAK_GBS, 4), traffic=traffic, kernel=dom,
                            avg_ms=kernels[dom]["ms"])
        if traffic:   # measured HBM bytes of the same kernel over the same duration (context for `frac`)
            roofline["measured_hbm_GBs"] = round(traffic / avg_s / 1e9, 1)
            roofline["measured_hbm_frac"] = round(traffic / avg_s / 1e9 / HBM_PEAK_GBS, 4)
        dr_ms = sum(kernels[n]["ms"] for n in DR_KERNELS if n in kernels)
        dr_flops = sum(models[n][1] for n in DR_KERNELS if n.startswith("dr_spmm"))
        dr_region = dict(kernels="D-ReLU x2 + DR-SpMM fwd x3 + bwd x3", sum_ms=round(dr_ms, 4),
                         MB=round(dr_bytes / 1e6, 1), GBs=round(dr_bytes / (dr_ms * 1e-3) / 1e9, 1),
                         frac_of_hbm_peak=round(dr_bytes / (dr_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                         GFLOPs=round(dr_flops / (dr_ms * 1e-3) / 1e9, 1))

    out = {
        "metric": "HeteroConv DR-SpMM fwd+bwd effective GB/s",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {g.Nc} cells, {g.Nn} nets, E_near={E['near']}, "
                               f"E_pins={E['pins']}, D={D}, k={klabel}, one HeteroConv layer fwd+bwd"
                               + (" (cell ids randomly permuted)" if args.permute_cells else ""),
                   "step_algorithmic_MB": round(step_bytes / 1e6, 1),
                   "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
                   "relation_overlap": args.overlap,
                   "setup_s": round(t_setup, 2), "context_create_s": round(t_ctx, 3)},
        "roofline": roofline,
        "dr_spmm_kernels": dr_region,
        "kernels": kernels,
    }
    if k_profile:
        out["k_profile"] = k_profile
    if not args.no_cpu_baseline:
        scale = args.cpu_scale or max(1, g.Nc // 200000)     # about 10-15 s of single-thread oracle work
        out["cpu_baseline"] = cpu_baseline(args.workload, D, ks, scale)
    layer.heteroconv_destroy()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
