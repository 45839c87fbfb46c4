"""Seeded synthetic circuit graphs and tensors shaped like CircuitNet designs.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds none of the method's arithmetic: it only draws random
graph *patterns* (CSR row pointers and column indices, no edge values), random
feature / weight / gradient tensors, and the list of named workloads.
"""
from .generate import (  # noqa: F401
    WORKLOADS,
    CircuitGraph,
    LayerTensors,
    block_diagonal,
    make_graph,
    make_tensors,
    workload,
)
