"""Parity of the whole layer at the benchmark's full size (1.2 M cells, 0.9 M nets, D = 128, k swept over 8, 16, 32,
64, the launch configuration bench.py times): sampled nodes against the oracle's layer on induced sub-problems, all
five weight gradients entry by entry (see sampled_checks.py); test_gpu_large_exhaustive.py compares every element of
the D-ReLU / DR-SpMM kernels at k = 32."""
import pytest

import sampled_checks as sc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def inputs():
    return sc.make_inputs("large")


@pytest.fixture(scope="module", params=[32, 8, 16, 64], ids=lambda k: f"k{k}")
def run(request, inputs):
    out = sc.run_layer(inputs, request.param)
    yield out
    out["layer"].heteroconv_destroy()


def test_large_setup_is_bit_exact(inputs):
    sc.check_setup(inputs)


def test_large_forward_sampled_rows(run):
    sc.check_forward(run)


def test_large_backward_sampled_rows(run):
    sc.check_backward(run)


def test_large_weight_gradients_sampled_entries_and_probe_identity(run):
    sc.check_weight_gradients(run)
