import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def tiny_graph():
    from circuit_synth import make_graph
    return make_graph("tiny", seed=0)


@pytest.fixture(scope="session")
def tiny_tensors():
    from circuit_synth import make_tensors, workload
    w = workload("tiny")
    return make_tensors(w["Nc"], w["Nn"], w["D"], seed=0)
