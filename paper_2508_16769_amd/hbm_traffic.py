"""Turn two rocprofv3 counter runs of `bench.py` into per-kernel HBM bytes.

rocprofv3 reports FETCH_SIZE and WRITE_SIZE in KiB per dispatch.  This tool attributes the dispatches of
the timed steps to the layer's kernels and writes `{workload.k: {kernel: bytes}}`, the table `bench.py`
reads for `roofline.traffic`.  The two counter runs must use the single-stream schedule, in which the
kernels of a step are dispatched in the fixed order listed in `SCHEDULE`:

    AMD_SERIALIZE_KERNEL=3 rocprofv3 --pmc FETCH_SIZE --kernel-trace -d <dir>/FETCH_SIZE -o bench \
        --output-format csv -- python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-profile-events \
        --overlap off
    (the same with WRITE_SIZE), then

    python3 -m paper_2508_16769_amd.hbm_traffic --fetch <dir>/FETCH_SIZE/bench_counter_collection.csv \
        --write <dir>/WRITE_SIZE/bench_counter_collection.csv --workload large --k 32

The counters are scaled by what the same counter reads for a plain device copy of known size
(`bench.py --copy-calibration` under the same rocprofv3 command): on MI355X FETCH_SIZE reads half the
bytes actually fetched (factor 2.0) and WRITE_SIZE reads them all (factor 1.0).
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os

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
HOT = ("topk_rows", "spmm_fwd", "spmm_bwd", "proj_kernel", "wgrad_partial", "wgrad_reduce")


def per_kernel_kib(path: str) -> dict:
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


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--fetch", required=True, help="counter_collection.csv of the FETCH_SIZE run")
    ap.add_argument("--write", required=True, help="counter_collection.csv of the WRITE_SIZE run")
    ap.add_argument("--workload", required=True)
    ap.add_argument("--k", type=int, required=True)
    ap.add_argument("--fetch-scale", type=float, default=2.0)
    ap.add_argument("--write-scale", type=float, default=1.0)
    ap.add_argument("--out", default=os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                                                   "profiles", "hbm_traffic.json"))
    args = ap.parse_args()
    f, w = per_kernel_kib(args.fetch), per_kernel_kib(args.write)
    table = {}
    print(f"{'kernel':26s} {'FETCH_SIZE KiB':>15s} {'WRITE_SIZE KiB':>15s} {'HBM MB':>10s}")
    for label, _ in SCHEDULE:
        b = (args.fetch_scale * f[label] + args.write_scale * w[label]) * 1024
        print(f"{label:26s} {f[label]:15.0f} {w[label]:15.0f} {b / 1e6:10.1f}")
        table[label] = round(b)
    allt = json.load(open(args.out)) if os.path.exists(args.out) else {}
    allt[f"{args.workload}.k{args.k}"] = table
    json.dump(allt, open(args.out, "w"), indent=1)
    print(f"wrote {args.out} [{args.workload}.k{args.k}]")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
