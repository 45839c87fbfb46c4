"""Times the multi-layer training step on a batch of synthetic sub-graphs: one stream per sub-graph against the
batch stacked into one block-diagonal graph.

    python3 -m paper_2508_16769_amd.train_profile [--workload subgraph] [--graphs 8] [--layers 3] [--steps 20] [--out table.md]

Prints a markdown table (wall-clock per step between device synchronisations, after three warm-up steps).
"""
from __future__ import annotations

import argparse
import os
import sys
import time

import numpy as np
import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import paper_2508_16769_amd as P  # noqa: E402
from circuit_synth import make_graph, workload  # noqa: E402


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="subgraph")
    ap.add_argument("--graphs", type=int, default=8)
    ap.add_argument("--layers", type=int, default=3)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
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
             f"Command: `python3 -m paper_2508_16769_amd.train_profile --workload {args.workload} --graphs {G} --layers {L} "
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


if __name__ == "__main__":
    raise SystemExit(main())
