"""The hot kernels keep nothing in scratch memory (checked on the compiler's own resource report, no GPU needed).

A scratch access is a vector-memory operation: the wavefront's wait for it also waits for every gather issued before
it, which once serialized the ping-pong batches of the DR-SpMM kernels (their per-group record stream had been placed
in scratch because one of its members was written on one side of a branch only)."""
import re
from concurrent.futures import ThreadPoolExecutor

from paper_2508_16769_amd import build


def _report():
    with ThreadPoolExecutor(max_workers=3) as pool:
        parts = list(pool.map(build.kernel_resources, ("topk.hip", "spmm.hip", "staged.hip")))
    out = {}
    for p in parts:
        out.update(p)
    return out


def test_hot_kernels_use_no_scratch_memory():
    rep = _report()
    topk = {k: v for k, v in rep.items() if "topk_rows_kernel" in k}
    spmm = {k: v for k, v in rep.items() if "spmm_fwd_kernel" in k or "spmm_bwd_kernel" in k}
    staged = {k: v for k, v in rep.items() if "spmm_bwd_staged_kernel" in k}
    assert len(topk) >= 10 and len(spmm) >= 20 and len(staged) >= 16
    for name, r in {**topk, **spmm}.items():
        assert r["ScratchSize"] == 0 and r["VGPRs Spill"] == 0, (name, r)
    # staged tiles: the instantiations with 64-column slabs and up to 4 compact outputs per lane (k <= 64) hold their two
    # prefetch sets in registers; the widest ones (8 outputs per lane, k up to 128) are allowed to spill
    for name, r in staged.items():
        m = re.search(r"staged_kernelILi(\d+)ELi(\d+)ELi(\d+)E", name)
        cw, ks = int(m.group(1)), int(m.group(2))
        if cw == 64 and ks <= 4:
            assert r["ScratchSize"] == 0 and r["VGPRs Spill"] == 0, (name, r)
    # the forward and backward kernels of the benchmark's width (k = 32) leave room for five wavefronts per SIMD or more
    for name, r in spmm.items():
        if "ILi4ELi2ELb0E" in name:
            assert r["Occupancy"] >= 5, (name, r)
