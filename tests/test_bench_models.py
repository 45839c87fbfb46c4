"""Host-side checks of bench.py's byte models and command line (no GPU)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402

# workload `large` at k = 32: node and edge counts of the seeded generator
NC, NN, D, K = 1_200_000, 900_000, 128, 32
E = dict(near=14_734_099, pins=6_900_281, pinned=6_900_281)


def test_dr_kernel_bytes_match_the_compulsory_byte_table():
    """Sum over the three relations of the compulsory bytes per direction, and the D-ReLU read / write volumes, against
    the figures tabulated for this workload (2 560 MB per direction, 1 080 MB read, 403 MB written)."""
    m = bench.operation_models(NC, NN, E, D, (K, K, K, K))
    fwd = sum(m[f"dr_spmm_fwd.{r}"][0] for r in ("near", "pins", "pinned"))
    bwd = sum(m[f"dr_spmm_bwd.{r}"][0] for r in ("near", "pins", "pinned"))
    assert fwd / 1e6 == pytest.approx(2560, rel=0.01)
    assert bwd / 1e6 == pytest.approx(2560, rel=0.01)
    topk = m["dr_topk.cell"][0] + m["dr_topk.net"][0]
    assert topk / 1e6 == pytest.approx(1080 + 403, rel=0.01)
    flops = sum(m[f"dr_spmm_fwd.{r}"][1] for r in ("near", "pins", "pinned"))
    assert flops / 1e6 == pytest.approx(2 * K * sum(E.values()) / 1e6)        # 2 E k per direction


def test_step_bytes_do_not_depend_on_kernel_fusion():
    ops = bench.operation_models(NC, NN, E, D, (K, K, K, K))
    ker = bench.kernel_models(NC, NN, E, D, (K, K, K, K))
    assert len(ops) == 21 and len(ker) == 19
    assert set(ker) - set(ops) == {"wgrad.near", "wgrad.pins"}
    # a paired weight-gradient kernel moves what its two operations move, minus one read of the shared upstream
    # gradient (and of its mask where there is one); the flops add up
    saved_near = ops["wgrad.neigh_near"][0] + ops["wgrad.self_near"][0] - ker["wgrad.near"][0]
    saved_pins = ops["wgrad.neigh_pins"][0] + ops["wgrad.self_pins"][0] - ker["wgrad.pins"][0]
    assert saved_near == 5 * NC * D and saved_pins == 4 * NN * D
    assert ker["wgrad.near"][1] == ops["wgrad.neigh_near"][1] + ops["wgrad.self_near"][1]
    for name in set(ker) & set(ops):
        assert ker[name] == ops[name]


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr) or "single" in (r.stdout + r.stderr).lower()
