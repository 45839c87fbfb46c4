#!/usr/bin/env python3
"""Secondary measurements of the library, each a sub-command that prints a markdown table (the summaries under
`profiles/` name the command that wrote them):

    python3 measure.py adaptive  ...   degree-adaptive K next to uniform K, per relation
    python3 measure.py train     ...   the multi-layer training step: one stream per sub-graph against the stacked batch
    python3 measure.py pipeline  ...   host-side pipeline against the per-graph path
    python3 measure.py overlap   ...   three relation streams against one: whole layer and the D-ReLU / DR-SpMM region
    python3 measure.py traffic   ...   rocprofv3 FETCH_SIZE / WRITE_SIZE runs of bench.py -> HBM bytes per kernel

`python3 measure.py <mode> --help` describes each.  The headline benchmark is `bench.py`.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _gpu_imports():
    global np, torch, P, make_graph, workload
    import numpy as np
    import torch
    import paper_2508_16769_amd as P
    from circuit_synth import make_graph, workload


def _time(fn, reps):
    """Mean milliseconds of fn over reps launches after three warm-ups (HIP events on the current stream)."""
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def mode_adaptive(argv) -> int:
    """Times the degree-adaptive-K kernels next to the uniform-K ones on the three relations of a synthetic workload.

    python3 measure.py adaptive [--workload large] [--k1 32 --k2 16 --k3 8] [--out table.md]

For each relation: `dr_topk` / `dr_topk_ranked`, `dr_spmm_fwd` / `dr_spmm_fwd_adaptive` and `dr_spmm_bwd` /
`dr_spmm_bwd_adaptive`, HIP events around `--reps` launches after three warm-ups.  The class boundaries are the
median and the 90th percentile of the relation's in-degrees.  Prints a markdown table."""
    ap = argparse.ArgumentParser(prog="measure.py adaptive", description=mode_adaptive.__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--k1", type=int, default=32)
    ap.add_argument("--k2", type=int, default=16)
    ap.add_argument("--k3", type=int, default=8)
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--out", default=None)
    args = ap.parse_args(argv)
    w = workload(args.workload)
    D = w["D"]
    g = make_graph(args.workload, seed=0)
    rng = np.random.default_rng(0)
    Xc = torch.from_numpy(rng.standard_normal((g.Nc, D)).astype(np.float32)).cuda()
    Xn = torch.from_numpy(rng.standard_normal((g.Nn, D)).astype(np.float32)).cuda()
    k1, k2, k3 = args.k1, args.k2, args.k3
    lines = [f"# Degree-adaptive K: DR-SpMM kernel times on the relations of workload `{args.workload}` (D = {D})", "",
             f"Command: `python3 measure.py adaptive --workload {args.workload} --k1 {k1} --k2 {k2} "
             f"--k3 {k3} --reps {args.reps}` (HIP events around {args.reps} launches after 3 warm-ups).",
             "Class boundaries t1, t2: median and 90th percentile of the relation's in-degrees.", "",
             "| relation | in-degree mean / p50 / p99 / max | kernels | fwd ms | bwd ms |", "|---|---|---|---|---|"]
    for name, pat, mode, Xs, Xd in (("near", g.near, P.DR_NORM_MEAN, Xc, Xc), ("pins", g.pins, P.DR_NORM_MEAN, Xc, Xn),
                                    ("pinned", g.pinned, P.DR_NORM_SYM, Xn, Xc)):
        A = P.device_relation(pat, mode)
        At = P.device_transpose(A)
        M, N = A.n_rows, A.n_cols
        deg = np.diff(pat.rowptr)
        degs = f"{deg.mean():.1f} / {np.median(deg):.0f} / {np.percentile(deg, 99):.0f} / {deg.max()}"
        H = torch.empty((M, D), device="cuda")
        tk = {}
        for k in sorted({k1, k2, k3}, reverse=True):
            v = torch.empty((N, k), device="cuda")
            i = torch.empty((N, k), dtype=torch.int16, device="cuda")
            G = torch.empty((N, k), device="cuda")
            tk[k] = _time(lambda: P.dr_topk(Xs, k, v, i), args.reps)
            f = _time(lambda: P.dr_spmm_fwd(A, v, i, D, k, H), args.reps)
            b = _time(lambda: P.dr_spmm_bwd(At, Xd, i, D, k, G), args.reps)
            lines.append(f"| {name} | {degs} | uniform K = {k} | {f:.3f} | {b:.3f} |")
        v = torch.empty((N, k1), device="cuda")
        i = torch.empty((N, k1), dtype=torch.int16, device="cuda")
        G = torch.empty((N, k1), device="cuda")
        t_ranked = _time(lambda: P.dr_topk_ranked(Xs, k1, v, i), args.reps)
        t1, t2 = int(np.percentile(deg, 50)), int(np.percentile(deg, 90))
        big = int(deg.max()) + 1
        for label, cls in ((f"adaptive, every row low ({k1})", (big, big, k1, k1, k1)),
                           (f"adaptive, t1 = {t1}, t2 = {t2}, widths ({k1}, {k2}, {k3})", (t1, t2, k1, k2, k3)),
                           (f"adaptive, every row high ({k3} of {k1} stored)", (0, 0, k1, k3, k3))):
            ecls = torch.empty(At.nnz, dtype=torch.uint8, device="cuda")
            P.dr_degree_edge_classes(At, A.rowptr, cls, ecls)
            f = _time(lambda: P.dr_spmm_fwd_adaptive(A, v, i, D, cls, H), args.reps)
            b = _time(lambda: P.dr_spmm_bwd_adaptive(At, ecls, Xd, i, D, cls, G), args.reps)
            if cls[0] == t1 and cls[1] == t2:
                e = [deg[deg <= t1].sum(), deg[(deg > t1) & (deg <= t2)].sum(), deg[deg > t2].sum()]
                label += " (edges per class " + ", ".join(f"{x / max(1, deg.sum()):.0%}" for x in e) + ")"
            lines.append(f"| {name} | {degs} | {label} | {f:.3f} | {b:.3f} |")
        lines.append(f"| {name} | | D-ReLU at K = {k1}: `dr_topk` {tk[k1]:.3f} ms, `dr_topk_ranked` {t_ranked:.3f} ms | | |")
        print("\n".join(lines[-8:]), flush=True)
    text = "\n".join(lines) + "\n"
    if args.out:
        with open(args.out, "w") as fh:
            fh.write(text)
    return 0


def mode_train(argv) -> int:
    """Times the multi-layer training step on a batch of synthetic sub-graphs: one stream per sub-graph against the
batch stacked into one block-diagonal graph.

    python3 measure.py train [--workload subgraph] [--graphs 8] [--layers 3] [--steps 20] [--out table.md]

Prints a markdown table (wall-clock per step between device synchronisations, after three warm-up steps)."""
    ap = argparse.ArgumentParser(prog="measure.py train", description=mode_train.__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="subgraph")
    ap.add_argument("--graphs", type=int, default=8)
    ap.add_argument("--layers", type=int, default=3)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--out", default=None)
    args = ap.parse_args(argv)
    w = workload(args.workload)
    D, k, L, G = w["D"], w["k"], args.layers, args.graphs
    gs = [make_graph(args.workload, seed=q) for q in range(G)]
    rng = np.random.default_rng(0)

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    keep = [(P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
             P.device_relation(g.pinned, P.DR_NORM_SYM)) for g in gs]
    ctxs = [P.HeteroConv(d[0], d[1], d[2], D, k, k) for d in keep]
    Nc, Nn = sum(g.Nc for g in gs), sum(g.Nn for g in gs)
    allc = dev(rng.standard_normal((Nc, D)).astype(np.float32))
    alln = dev(rng.standard_normal((Nn, D)).astype(np.float32))
    allt = dev(rng.standard_normal(Nc).astype(np.float32))
    oc = np.cumsum([0] + [g.Nc for g in gs])
    on = np.cumsum([0] + [g.Nn for g in gs])
    Xc = [allc[oc[q]:oc[q + 1]] for q in range(G)]
    Xn = [alln[on[q]:on[q + 1]] for q in range(G)]
    tg = [allt[oc[q]:oc[q + 1]] for q in range(G)]
    Xc_s = [t.clone() for t in Xc]                       # the same inputs, scattered in memory
    Xn_s = [t.clone() for t in Xn]
    tg_s = [t.clone() for t in tg]
    n = P.hgnn_num_params(L, D)
    theta0 = rng.uniform(-0.15, 0.15, n).astype(np.float32)

    def run(batched, xs):
        model = P.Hgnn(ctxs, L, batched=batched)
        th, m, v = dev(theta0), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
        gr, ls = torch.empty(n, device="cuda"), torch.empty(1, device="cuda")
        for i in range(3):
            model.hgnn_train_step(xs[0], xs[1], xs[2], th, m, v, 2e-4, .9, .999, 1e-8, 1e-5, 1 + i, gr, ls)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            model.hgnn_train_step(xs[0], xs[1], xs[2], th, m, v, 2e-4, .9, .999, 1e-8, 1e-5, 4 + i, gr, ls)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        loss = float(ls.cpu()[0])
        model.hgnn_destroy()
        return dt, loss

    rows = [("one stream and one enqueueing host thread per sub-graph (`hgnn_create`)", run(False, (Xc_s, Xn_s, tg_s))),
            ("stacked into one block-diagonal graph (`hgnn_create_batched`), inputs gathered each step", run(True, (Xc_s, Xn_s, tg_s))),
            ("stacked, inputs already behind one another in memory (read in place)", run(True, (Xc, Xn, tg)))]
    lines = [f"# Training step on {G} sub-graphs of workload `{args.workload}` ({L} layers, D = {D}, k = {k})", "",
             f"Command: `python3 measure.py train --workload {args.workload} --graphs {G} --layers {L} "
             f"--steps {args.steps}`.",
             f"Per sub-graph: {gs[0].Nc} cells, {gs[0].Nn} nets, {gs[0].near.nnz} near and {gs[0].pins.nnz} pins edges.  "
             f"Forward, read-out, MSE, backward and Adam of all sub-graphs = one step.", "",
             "| batch mapping | ms per step | loss after the timed steps |", "|---|---|---|"]
    for name, (dt, loss) in rows:
        lines.append(f"| {name} | {dt * 1e3:.2f} | {loss:.5f} |")
    text = "\n".join(lines) + "\n"
    print(text, flush=True)
    if args.out:
        with open(args.out, "w") as fh:
            fh.write(text)
    for c in ctxs:
        c.heteroconv_destroy()
    return 0


def mode_pipeline(argv) -> int:
    """Times a stream of host-resident sub-graphs through (a) the ordinary per-graph path and (b) the host-side pipeline.

    python3 measure.py pipeline [--workload subgraph] [--graphs 24] [--layers 3] [--out table.md]

Every sub-graph arrives as host arrays (two CSR patterns and two embedding matrices).  The GPU work per sub-graph is
`--layers` HeteroConv forward + backward passes.  (a) uploads with blocking copies, builds a context (device
allocations, edge values, transposes), computes, waits and frees, one sub-graph after the other.  (b) runs the same
kernels through dr_pipeline_*: worker threads stage and upload the next sub-graphs and enqueue their setup on their
own streams while the GPU computes; the consumer never waits for the GPU until the end.  Prints a markdown table."""
    ap = argparse.ArgumentParser(prog="measure.py pipeline", description=mode_pipeline.__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="subgraph")
    ap.add_argument("--graphs", type=int, default=24)
    ap.add_argument("--distinct", type=int, default=8, help="distinct sub-graphs generated (the stream cycles through them)")
    ap.add_argument("--layers", type=int, default=3)
    ap.add_argument("--out", default=None)
    args = ap.parse_args(argv)
    w = workload(args.workload)
    D, k = w["D"], w["k"]
    rng = np.random.default_rng(0)
    gs = [make_graph(args.workload, seed=q) for q in range(args.distinct)]
    feats = [(rng.standard_normal((g.Nc, D)).astype(np.float32), rng.standard_normal((g.Nn, D)).astype(np.float32)) for g in gs]
    Nc, Nn = max(g.Nc for g in gs), max(g.Nn for g in gs)
    W = {n: torch.from_numpy(rng.uniform(-0.15, 0.15, (D, D)).astype(np.float32)).cuda() for n in P.WEIGHT_NAMES}
    dYc = torch.from_numpy(rng.standard_normal((Nc, D)).astype(np.float32)).cuda()
    dYn = torch.from_numpy(rng.standard_normal((Nn, D)).astype(np.float32)).cuda()
    Yc, Yn = torch.empty_like(dYc), torch.empty_like(dYn)
    dXc, dXn = torch.empty_like(dYc), torch.empty_like(dYn)
    dW = {n: torch.empty((D, D), device="cuda") for n in P.WEIGHT_NAMES}
    stream = torch.cuda.current_stream()

    def compute(layer, xc, xn, saved):
        for _ in range(args.layers):
            layer.heteroconv_fwd(xc, xn, W, Yc, Yn, saved)
            layer.heteroconv_bwd(dYc, dYn, W, saved, dXc, dXn, dW)

    def ordinary():
        t0 = time.perf_counter()
        for i in range(args.graphs):
            g, (xc_h, xn_h) = gs[i % len(gs)], feats[i % len(gs)]
            rel = (P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN),
                   P.device_relation(g.pinned, P.DR_NORM_SYM))
            layer = P.HeteroConv(*rel, D, k, k)
            saved = layer.alloc_saved()
            compute(layer, torch.from_numpy(xc_h).cuda(), torch.from_numpy(xn_h).cuda(), saved)
            torch.cuda.synchronize()
            layer.heteroconv_destroy()
        return time.perf_counter() - t0

    def pipelined(n_slots, n_threads):
        pl = P.Pipeline(n_slots, n_threads, Nc, Nn, max(g.near.nnz for g in gs), max(g.pins.nnz for g in gs), D, k, k)
        saved = None
        torch.cuda.synchronize()
        t0 = time.perf_counter()

        def submit(i):
            g, (xc_h, xn_h) = gs[i % len(gs)], feats[i % len(gs)]
            pl.dr_pipeline_submit(i % n_slots, g.near.rowptr, g.near.colidx, g.pins.rowptr, g.pins.colidx, xc_h, xn_h)

        for i in range(min(n_slots, args.graphs)):
            submit(i)
        for i in range(args.graphs):
            slot = i % n_slots
            layer, xc, xn = pl.dr_pipeline_acquire(slot, stream)
            if saved is None:
                saved = layer.alloc_saved()
            compute(layer, xc, xn, saved)
            pl.dr_pipeline_release(slot, stream)
            if i + n_slots < args.graphs:
                submit(i + n_slots)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        pl.dr_pipeline_destroy()
        return dt

    def compute_only():
        g, (xc_h, xn_h) = gs[0], feats[0]
        rel = (P.device_relation(g.near, P.DR_NORM_MEAN), P.device_relation(g.pins, P.DR_NORM_MEAN), P.device_relation(g.pinned, P.DR_NORM_SYM))
        layer = P.HeteroConv(*rel, D, k, k)
        saved = layer.alloc_saved()
        xc, xn = torch.from_numpy(xc_h).cuda(), torch.from_numpy(xn_h).cuda()
        compute(layer, xc, xn, saved)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.graphs):
            compute(layer, xc, xn, saved)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        layer.heteroconv_destroy()
        return dt

    ordinary()                                   # warm-up: allocator, kernels
    rows = [("GPU work alone (graph already resident, no setup)", compute_only())]
    rows.append(("ordinary path, one sub-graph after the other", ordinary()))
    for n_slots, n_threads in ((1, 1), (2, 2), (3, 3), (4, 4)):
        pipelined(n_slots, n_threads)            # warm-up
        rows.append((f"pipeline, {n_slots} slot(s), {n_threads} worker thread(s)", pipelined(n_slots, n_threads)))
    base = rows[1][1]
    mb = sum(4 * (g.near.nnz + g.pins.nnz + g.Nc + g.Nn + 2) + 4 * D * (g.Nc + g.Nn) for g in gs) / len(gs) / 1e6
    lines = [f"# Host-side pipeline: {args.graphs} sub-graphs of workload `{args.workload}` streamed from host memory", "",
             f"Command: `python3 measure.py pipeline --workload {args.workload} --graphs {args.graphs} "
             f"--layers {args.layers}`.",
             f"Per sub-graph: {gs[0].Nc} cells, {gs[0].Nn} nets, D = {D}, k = {k}; {mb:.1f} MB uploaded; GPU work = {args.layers} x "
             f"(heteroconv_fwd + heteroconv_bwd).  Host: {len(os.sched_getaffinity(0))} cores available.", "",
             "| mode | total ms | ms per sub-graph | saving vs the ordinary path |", "|---|---|---|---|"]
    for name, dt in rows:
        lines.append(f"| {name} | {dt * 1e3:.1f} | {dt * 1e3 / args.graphs:.2f} | {(1 - dt / base) * 100:.1f} % |")
    text = "\n".join(lines) + "\n"
    print(text, flush=True)
    if args.out:
        with open(args.out, "w") as fh:
            fh.write(text)
    return 0


# (label, substring the dispatched kernel's name must contain) in single-stream dispatch order of one
# forward + backward step
SCHEDULE = (
    ("dr_topk.net", "topk_rows"), ("dr_spmm_fwd.pinned", "spmm_fwd"),
    ("dr_topk.cell", "topk_rows"), ("dr_spmm_fwd.pins", "spmm_fwd"), ("dr_spmm_fwd.near", "spmm_fwd"),
    ("proj.near", "proj_kernel"), ("proj.pins", "proj_kernel"), ("proj.pinned+merge", "proj_kernel"),
    ("dproj.near", "proj_kernel"), ("dr_spmm_bwd.near", "spmm_bwd"),
    ("wgrad.near", "wgrad_partial"), ("wgrad.near.reduce_neigh", "wgrad_reduce"), ("wgrad.near.reduce_self", "wgrad_reduce"),
    ("dproj.pins", "proj_kernel"), ("dr_spmm_bwd.pins", "spmm_bwd"),
    ("dself.near+dX", "proj_kernel"),
    ("wgrad.pins", "wgrad_partial"), ("wgrad.pins.reduce_neigh", "wgrad_reduce"), ("wgrad.pins.reduce_self", "wgrad_reduce"),
    ("dproj.pinned", "proj_kernel"), ("dr_spmm_bwd.pinned", "spmm_bwd"),
    ("dself.pins+dX", "proj_kernel"),
    ("wgrad.pinned", "wgrad_partial"), ("wgrad.pinned.reduce", "wgrad_reduce"),
)
# single-stream dispatch order of `bench.py --only dr --serial` (the timed D-ReLU / DR-SpMM region alone)
SCHEDULE_DR = (
    ("dr_topk.cell", "topk_rows"), ("dr_spmm_fwd.near", "spmm_fwd"), ("dr_spmm_bwd.near", "spmm_bwd"),
    ("dr_spmm_fwd.pins", "spmm_fwd"), ("dr_spmm_bwd.pins", "spmm_bwd"),
    ("dr_topk.net", "topk_rows"), ("dr_spmm_fwd.pinned", "spmm_fwd"), ("dr_spmm_bwd.pinned", "spmm_bwd"),
)
HOT = ("topk_rows", "spmm_fwd", "spmm_bwd", "proj_kernel", "wgrad_partial", "wgrad_reduce")


def per_kernel_kib(path: str, SCHEDULE=SCHEDULE) -> dict:
    """Mean counter value per schedule label over the timed steps (the first step is warm-up)."""
    rows = list(csv.DictReader(open(path, newline="")))
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    hot = [r for r in rows if any(s in r["Kernel_Name"] for s in HOT)]
    n = len(SCHEDULE)
    if len(hot) % n or len(hot) < 2 * n:
        raise SystemExit(f"{path}: {len(hot)} hot dispatches is not a multiple (>= 2) of the {n}-kernel schedule")
    acc = collections.defaultdict(list)
    for i, r in enumerate(hot):
        label, pat = SCHEDULE[i % n]
        if pat not in r["Kernel_Name"]:
            raise SystemExit(f"{path}: dispatch {r['Dispatch_Id']} is {r['Kernel_Name'][:60]!r}, expected {pat} "
                             f"for {label}: the run did not use the single-stream schedule")
        if i >= n:
            acc[label].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in acc.items()}


def mode_traffic(argv) -> int:
    """Turn two rocprofv3 counter runs of `bench.py` into per-kernel HBM bytes.

rocprofv3 reports FETCH_SIZE and WRITE_SIZE in KiB per dispatch.  This tool attributes the dispatches of
the timed steps to the layer's kernels and writes `{workload.k: {kernel: bytes}}`, the table `bench.py`
reads for `roofline.traffic`.  The two counter runs must use the single-stream schedule, in which the
kernels of a step are dispatched in the fixed order listed in `SCHEDULE`:

    AMD_SERIALIZE_KERNEL=3 rocprofv3 --pmc FETCH_SIZE --kernel-trace -d <dir>/FETCH_SIZE -o bench \
        --output-format csv -- python3 bench.py --only layer --steps 3 --warmup 1 --no-cpu-baseline \
        --no-profile-events --overlap off
    (the same with WRITE_SIZE), then

    python3 measure.py traffic --fetch <dir>/FETCH_SIZE/bench_counter_collection.csv \
        --write <dir>/WRITE_SIZE/bench_counter_collection.csv --workload large --k 32

The counters are scaled by what the same counter reads for a plain device copy of known size
(`bench.py --copy-calibration` under the same rocprofv3 command): on MI355X FETCH_SIZE reads half the
bytes actually fetched (factor 2.0) and WRITE_SIZE reads them all (factor 1.0)."""
    ap = argparse.ArgumentParser(prog="measure.py traffic", description=mode_traffic.__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--fetch", required=True, help="counter_collection.csv of the FETCH_SIZE run")
    ap.add_argument("--write", required=True, help="counter_collection.csv of the WRITE_SIZE run")
    ap.add_argument("--workload", required=True)
    ap.add_argument("--k", type=int, required=True)
    ap.add_argument("--schedule", choices=("layer", "dr"), default="layer",
                    help="layer: `bench.py --only layer --overlap off`; dr: `bench.py --only dr --serial`")
    ap.add_argument("--measured", default=None, help="note stored with the table (date, commit, command)")
    ap.add_argument("--fetch-scale", type=float, default=2.0)
    ap.add_argument("--write-scale", type=float, default=1.0)
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles", "hbm_traffic.json"))
    args = ap.parse_args(argv)
    sched = SCHEDULE if args.schedule == "layer" else SCHEDULE_DR
    f, w = per_kernel_kib(args.fetch, sched), per_kernel_kib(args.write, sched)
    table = {}
    print(f"{'kernel':26s} {'FETCH_SIZE KiB':>15s} {'WRITE_SIZE KiB':>15s} {'HBM MB':>10s}")
    for label, _ in sched:
        b = (args.fetch_scale * f[label] + args.write_scale * w[label]) * 1024
        print(f"{label:26s} {f[label]:15.0f} {w[label]:15.0f} {b / 1e6:10.1f}")
        table[label] = round(b)
    allt = json.load(open(args.out)) if os.path.exists(args.out) else {}
    key = f"{args.workload}.k{args.k}"
    allt.setdefault(key, {}).update(table)
    if args.measured:
        allt.setdefault("measured", {})[key] = args.measured
    json.dump(allt, open(args.out, "w"), indent=1)
    print(f"wrote {args.out} [{args.workload}.k{args.k}]")
    return 0

def mode_overlap(argv) -> int:
    """Relation concurrency (paper Section 3.4): the three relations on three HIP streams against one stream, for the whole
    layer (heteroconv_fwd + heteroconv_bwd) and for the D-ReLU / DR-SpMM region of bench.py alone.

        python3 measure.py overlap [--workloads small,medium,large] [--steps 30] [--out table.md]

    Wall-clock per step between device synchronisations after five warm-up steps; two alternating rounds per schedule, the
    lower one reported."""
    import bench
    ap = argparse.ArgumentParser(prog="measure.py overlap", description=mode_overlap.__doc__,
                                 formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workloads", default="small,medium,large")
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--out", default=None)
    args = ap.parse_args(argv)
    from circuit_synth import make_tensors
    lines = ["# Relation concurrency: three streams against one", "",
             f"Command: `python3 measure.py overlap --workloads {args.workloads} --steps {args.steps}`.", "",
             "| workload | layer step, one stream ms | layer step, three streams ms | ratio | DR region, one stream ms | DR region, three streams ms | ratio |",
             "|---|---|---|---|---|---|---|"]
    for name in args.workloads.split(","):
        w = workload(name)
        D, k = w["D"], w["k"]
        g = make_graph(name, seed=0)
        T = make_tensors(g.Nc, g.Nn, D, seed=0)
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        rel = dict(near=P.device_relation(g.near, P.DR_NORM_MEAN), pins=P.device_relation(g.pins, P.DR_NORM_MEAN),
                   pinned=P.device_relation(g.pinned, P.DR_NORM_SYM))
        rel_t = {r: P.device_transpose(rel[r]) for r in rel}
        X = dict(cell=dev(T.X_cell), net=dev(T.X_net))
        dY = dict(cell=dev(T.dY_cell), net=dev(T.dY_net))
        layer = P.HeteroConv(rel["near"], rel["pins"], rel["pinned"], D, k, k)
        layer.heteroconv_set_cell_order(dev(g.cell_order))           # as bench.py: transposed near on LDS-staged tiles
        near_plan = P.SpmmPlan(rel_t["near"], D, dev(g.cell_order))
        saved = layer.alloc_saved()
        Wd = {n: dev(T.W[n]) for n in P.WEIGHT_NAMES}
        Yc = torch.empty((g.Nc, D), device="cuda")
        Yn = torch.empty((g.Nn, D), device="cuda")
        dXc, dXn = torch.empty_like(Yc), torch.empty_like(Yn)
        dW = {n: torch.empty((D, D), device="cuda") for n in P.WEIGHT_NAMES}

        def layer_ms(mode):
            layer.heteroconv_set_overlap(mode)
            for i in range(5 + args.steps):
                if i == 5:
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                layer.heteroconv_fwd(X["cell"], X["net"], Wd, Yc, Yn, saved)
                layer.heteroconv_bwd(dY["cell"], dY["net"], Wd, saved, dXc, dXn, dW)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / args.steps

        region = bench.DrRegion(P, torch, rel, rel_t, X, dY, D, k, near_plan)
        l1 = min(layer_ms(P.DR_OVERLAP_OFF) for _ in range(1))
        l3 = layer_ms(P.DR_OVERLAP_ON)
        l1 = min(l1, layer_ms(P.DR_OVERLAP_OFF))
        l3 = min(l3, layer_ms(P.DR_OVERLAP_ON))
        r1 = region.time_region(5, args.steps, concurrent=False)[0]
        r3 = region.time_region(5, args.steps, concurrent=True)[0]
        r1 = min(r1, region.time_region(5, args.steps, concurrent=False)[0])
        r3 = min(r3, region.time_region(5, args.steps, concurrent=True)[0])
        lines.append(f"| {name} ({g.Nc} cells, D = {D}, k = {k}) | {l1:.3f} | {l3:.3f} | {l1 / l3:.2f}x | {r1:.3f} | {r3:.3f} | {r1 / r3:.2f}x |")
        print(lines[-1], flush=True)
        layer.heteroconv_destroy()
        del region, layer, saved
    text = "\n".join(lines) + "\n"
    print(text, flush=True)
    if args.out:
        with open(args.out, "w") as fh:
            fh.write(text)
    return 0


MODES = {"overlap": mode_overlap, "adaptive": mode_adaptive, "train": mode_train, "pipeline": mode_pipeline, "traffic": mode_traffic}


def main() -> int:
    if len(sys.argv) < 2 or sys.argv[1] not in MODES:
        print(__doc__, file=sys.stderr)
        return 2
    if sys.argv[1] != "traffic":
        _gpu_imports()
    return MODES[sys.argv[1]](sys.argv[2:])


if __name__ == "__main__":
    raise SystemExit(main())
