"""Parity on the medium configuration (250 000 cells, 180 000 nets with 0.1 % high-fanout nets, D = 128, k = 32); see sampled_checks.py for how single outputs are recomputed."""
import pytest

import sampled_checks as sc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def inputs():
    return sc.make_inputs("medium")


@pytest.fixture(scope="module", params=[32], ids=lambda k: f"k{k}")
def run(request, inputs):
    out = sc.run_layer(inputs, request.param)
    yield out
    out["layer"].heteroconv_destroy()


def test_medium_setup_is_bit_exact(inputs):
    sc.check_setup(inputs)


def test_medium_forward_sampled_rows(run):
    sc.check_forward(run)


def test_medium_backward_sampled_rows(run):
    sc.check_backward(run)


def test_medium_weight_gradients_sampled_entries_and_probe_identity(run):
    sc.check_weight_gradients(run)
