"""Times the degree-adaptive-K kernels next to the uniform-K ones on the three relations of a synthetic workload.

    python3 -m paper_2508_16769_amd.adaptive_profile [--workload large] [--k1 32 --k2 16 --k3 8] [--out table.md]

For each relation: `dr_topk` / `dr_topk_ranked`, `dr_spmm_fwd` / `dr_spmm_fwd_adaptive` and `dr_spmm_bwd` /
`dr_spmm_bwd_adaptive`, HIP events around `--reps` launches after three warm-ups.  The class boundaries are the
median and the 90th percentile of the relation's in-degrees.  Prints a markdown table.
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np
import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import paper_2508_16769_amd as P  # noqa: E402
from circuit_synth import make_graph, workload  # noqa: E402


def _time(fn, reps):
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


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--k1", type=int, default=32)
    ap.add_argument("--k2", type=int, default=16)
    ap.add_argument("--k3", type=int, default=8)
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    w = workload(args.workload)
    D = w["D"]
    g = make_graph(args.workload, seed=0)
    rng = np.random.default_rng(0)
    Xc = torch.from_numpy(rng.standard_normal((g.Nc, D)).astype(np.float32)).cuda()
    Xn = torch.from_numpy(rng.standard_normal((g.Nn, D)).astype(np.float32)).cuda()
    k1, k2, k3 = args.k1, args.k2, args.k3
    lines = [f"# Degree-adaptive K: DR-SpMM kernel times on the relations of workload `{args.workload}` (D = {D})", "",
             f"Command: `python3 -m paper_2508_16769_amd.adaptive_profile --workload {args.workload} --k1 {k1} --k2 {k2} "
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


if __name__ == "__main__":
    raise SystemExit(main())
