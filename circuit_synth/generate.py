"""Seeded generators for CircuitNet-shaped heterogeneous graphs and layer tensors.

Two node types (cell, net) and three relations, as in the paper's Section 2.2:

* ``near``   cell -> cell, geometric links inside a spatial window (rows = destination cells)
* ``pins``   cell -> net,  topological links (rows = destination nets, columns = member cells)
* ``pinned`` net -> cell,  the exact transpose pattern of ``pins`` (rows = destination cells)

Only the sparsity *patterns* are produced here (row pointers and column
indices); edge values are part of the method (mean / symmetric normalisation)
and are computed by whoever consumes the pattern.  All index arrays are int32,
all tensors float32, and everything is a pure function of ``(workload, seed)``.

Random streams: every purpose has its own ``numpy`` PCG64 generator seeded with
``SeedSequence([seed, purpose_id])`` so tensors can be redrawn without
regenerating the graph.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

_STREAM_NEAR = 1
_STREAM_NET_DEGREE = 2
_STREAM_NET_MEMBERS = 3
_STREAM_X_CELL = 4
_STREAM_X_NET = 5
_STREAM_WEIGHTS = 6
_STREAM_UPSTREAM = 7
_STREAM_PERMUTE = 8


def _rng(seed: int, purpose: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), int(purpose)])))


# --------------------------------------------------------------------------
# workload table
# --------------------------------------------------------------------------

# near_law: ("const", d) | ("poisson", lam) | ("powerlaw", alpha, dmin, dmax)
# net_mean: mean of the geometric part G (degree = 2 + G, G on {1,2,...})
# net_cap : cap on the ordinary net degree (None = uncapped)
# evil    : fraction of nets (chosen uniformly) whose degree is uniform on [200, 2000]
WORKLOADS: Dict[str, dict] = {
    "tiny": dict(Nc=2048, Nn=1024, grid=(64, 32), near_law=("const", 8),
                 net_mean=3.0, net_cap=32, evil=0.0, D=64, k=16),
    "small": dict(Nc=60_000, Nn=40_000, grid=(300, 200), near_law=("poisson", 10.0),
                  net_mean=3.0, net_cap=64, evil=0.0, D=64, k=16),
    "medium": dict(Nc=250_000, Nn=180_000, grid=(500, 500), near_law=("poisson", 12.0),
                   net_mean=3.5, net_cap=None, evil=0.001, D=128, k=32),
    "large": dict(Nc=1_200_000, Nn=900_000, grid=(1200, 1000), near_law=("powerlaw", 2.2, 4, 256),
                  net_mean=3.5, net_cap=None, evil=0.002, D=128, k=32),
    "subgraph": dict(Nc=20_000, Nn=14_000, grid=(200, 100), near_law=("poisson", 10.0),
                     net_mean=3.0, net_cap=64, evil=0.0, D=128, k=32),
}


def workload(name: str) -> dict:
    """Return a copy of the named workload description."""
    return dict(WORKLOADS[name])


# --------------------------------------------------------------------------
# containers
# --------------------------------------------------------------------------

@dataclass
class Pattern:
    """CSR sparsity pattern: rows are destination nodes, columns are source nodes."""
    n_rows: int
    n_cols: int
    rowptr: np.ndarray  # int32 [n_rows + 1]
    colidx: np.ndarray  # int32 [nnz], ascending inside each row, no duplicates

    @property
    def nnz(self) -> int:
        return int(self.colidx.shape[0])


@dataclass
class CircuitGraph:
    name: str
    seed: int
    Nc: int
    Nn: int
    near: Pattern     # Nc x Nc
    pins: Pattern     # Nn x Nc
    pinned: Pattern   # Nc x Nn  (transpose pattern of pins)
    cell_order: Optional[np.ndarray] = None   # int32 [Nc]: the cells sorted along a Z-order curve of their placement


@dataclass
class LayerTensors:
    D: int
    X_cell: np.ndarray   # [Nc, D]
    X_net: np.ndarray    # [Nn, D]
    # Y = X @ W convention, every matrix [D, D]
    W: Dict[str, np.ndarray] = field(default_factory=dict)  # self_near, neigh_near, self_pins, neigh_pins, pinned
    dY_cell: Optional[np.ndarray] = None  # [Nc, D]
    dY_net: Optional[np.ndarray] = None   # [Nn, D]


WEIGHT_NAMES: Tuple[str, ...] = ("self_near", "neigh_near", "self_pins", "neigh_pins", "pinned")


# --------------------------------------------------------------------------
# degree laws
# --------------------------------------------------------------------------

def _near_degrees(law: tuple, n: int, rng: np.random.Generator) -> np.ndarray:
    kind = law[0]
    if kind == "const":
        return np.full(n, int(law[1]), dtype=np.int64)
    if kind == "poisson":
        return rng.poisson(float(law[1]), size=n).astype(np.int64)
    if kind == "powerlaw":
        alpha, dmin, dmax = float(law[1]), int(law[2]), int(law[3])
        support = np.arange(dmin, dmax + 1, dtype=np.float64)
        pmf = support ** (-alpha)
        cdf = np.cumsum(pmf / pmf.sum())
        cdf[-1] = 1.0
        u = rng.random(n)
        return (np.searchsorted(cdf, u, side="right") + dmin).astype(np.int64)
    raise ValueError(f"unknown near-degree law {law!r}")


def _net_degrees(n: int, mean_g: float, cap: Optional[int], evil: float,
                 rng: np.random.Generator) -> np.ndarray:
    deg = 2 + rng.geometric(1.0 / mean_g, size=n).astype(np.int64)
    if cap is not None:
        deg = np.minimum(deg, cap)
    n_evil = int(round(evil * n))
    if n_evil > 0:
        who = rng.choice(n, size=n_evil, replace=False)
        deg[who] = rng.integers(200, 2001, size=n_evil)
    return deg


# --------------------------------------------------------------------------
# relations
# --------------------------------------------------------------------------

def _csr_from_sorted(rows: np.ndarray, cols: np.ndarray, n_rows: int, n_cols: int) -> Pattern:
    counts = np.bincount(rows, minlength=n_rows)
    rowptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    assert rowptr[-1] < 2 ** 31
    return Pattern(n_rows, n_cols, rowptr.astype(np.int32), cols.astype(np.int32))


def _make_near(Nc: int, grid: Tuple[int, int], law: tuple, rng: np.random.Generator) -> Pattern:
    """Each destination cell draws ``d`` distinct source cells uniformly from the
    (2r+1)^2 window around it (clipped to the grid, itself excluded), with
    r = max(2, ceil(sqrt(d+1)) - 1) so that even a corner cell has d candidates."""
    W, H = grid
    assert W * H >= Nc
    deg = _near_degrees(law, Nc, rng)
    radius = np.maximum(2, np.ceil(np.sqrt(deg + 1.0)).astype(np.int64) - 1)
    out_rows, out_cols = [], []
    for r in np.unique(radius):
        ids = np.nonzero((radius == r) & (deg > 0))[0]
        if ids.size == 0:
            continue
        side = 2 * int(r) + 1
        dx = np.tile(np.arange(-r, r + 1), side)
        dy = np.repeat(np.arange(-r, r + 1), side)
        not_self = ~((dx == 0) & (dy == 0))
        chunk = max(1, (4 << 20) // (side * side))
        for s in range(0, ids.size, chunk):
            cid = ids[s:s + chunk]
            d = deg[cid]
            x = cid % W
            y = cid // W
            nx = x[:, None] + dx[None, :]
            ny = y[:, None] + dy[None, :]
            nid = ny * W + nx
            valid = (nx >= 0) & (nx < W) & (ny >= 0) & (ny < H) & (nid < Nc) & not_self[None, :]
            keys = rng.random(nid.shape)
            keys[~valid] = 2.0
            order = np.argsort(keys, axis=1, kind="stable")
            assert np.all(valid.sum(axis=1) >= d), "window too small for the requested degree"
            take = np.arange(side * side)[None, :] < d[:, None]
            chosen = np.take_along_axis(nid, order, axis=1)[take]
            out_rows.append(np.repeat(cid, d))
            out_cols.append(chosen)
    if out_rows:
        rows = np.concatenate(out_rows)
        cols = np.concatenate(out_cols)
    else:
        rows = np.zeros(0, dtype=np.int64)
        cols = np.zeros(0, dtype=np.int64)
    order = np.argsort(rows * np.int64(Nc) + cols, kind="stable")
    return _csr_from_sorted(rows[order], cols[order], Nc, Nc)


def _make_pins(Nn: int, Nc: int, mean_g: float, cap: Optional[int], evil: float,
               rng_deg: np.random.Generator, rng_mem: np.random.Generator) -> Pattern:
    """Rows are nets; each net's members are distinct uniformly random cells."""
    deg = _net_degrees(Nn, mean_g, cap, evil, rng_deg)
    deg = np.minimum(deg, Nc)
    rows = np.repeat(np.arange(Nn, dtype=np.int64), deg)
    cols = rng_mem.integers(0, Nc, size=rows.size, dtype=np.int64)
    while True:
        key = rows * np.int64(Nc) + cols
        order = np.argsort(key, kind="stable")
        rows, cols, key = rows[order], cols[order], key[order]
        dup = np.nonzero(key[1:] == key[:-1])[0] + 1
        if dup.size == 0:
            break
        cols[dup] = rng_mem.integers(0, Nc, size=dup.size, dtype=np.int64)
    return _csr_from_sorted(rows, cols, Nn, Nc)


def placement_order(Nc: int, grid: Tuple[int, int]) -> np.ndarray:
    """The cells sorted along the Z-order (Morton) curve of their placement coordinates (cell id = y * W + x): any run
    of 64 consecutive cells of this order covers a compact patch of the layout (an 8 x 8 square where the run is
    aligned).  A processing-order hint for kernels that stage the neighbourhood of a block of cells; it carries no
    arithmetic and changes no result."""
    W, _ = grid
    ids = np.arange(Nc, dtype=np.int64)

    def spread(v):
        v = v.astype(np.uint64)
        v = (v | (v << np.uint64(8))) & np.uint64(0x00FF00FF)
        v = (v | (v << np.uint64(4))) & np.uint64(0x0F0F0F0F)
        v = (v | (v << np.uint64(2))) & np.uint64(0x33333333)
        v = (v | (v << np.uint64(1))) & np.uint64(0x55555555)
        return v

    key = spread(ids % W) | (spread(ids // W) << np.uint64(1))
    return np.argsort(key, kind="stable").astype(np.int32)


def transpose_pattern(p: Pattern) -> Pattern:
    """Pattern of the transposed relation (index bookkeeping only, no values)."""
    rows = np.repeat(np.arange(p.n_rows, dtype=np.int64), np.diff(p.rowptr.astype(np.int64)))
    cols = p.colidx.astype(np.int64)
    order = np.argsort(cols * np.int64(p.n_rows) + rows, kind="stable")
    return _csr_from_sorted(cols[order], rows[order], p.n_cols, p.n_rows)


def permute_cells(g: CircuitGraph, seed: int = 0) -> CircuitGraph:
    """Same graph with the cell ids randomly relabelled (destroys the grid locality of
    ``near``); used only for the locality-sensitivity measurement."""
    perm = _rng(seed, _STREAM_PERMUTE).permutation(g.Nc).astype(np.int64)

    def relabel(p: Pattern, rows_are_cells: bool, cols_are_cells: bool) -> Pattern:
        rows = np.repeat(np.arange(p.n_rows, dtype=np.int64), np.diff(p.rowptr.astype(np.int64)))
        cols = p.colidx.astype(np.int64)
        if rows_are_cells:
            rows = perm[rows]
        if cols_are_cells:
            cols = perm[cols]
        order = np.argsort(rows * np.int64(p.n_cols) + cols, kind="stable")
        return _csr_from_sorted(rows[order], cols[order], p.n_rows, p.n_cols)

    order = None if g.cell_order is None else perm[g.cell_order.astype(np.int64)].astype(np.int32)
    return CircuitGraph(g.name + "-permuted", g.seed, g.Nc, g.Nn,
                        relabel(g.near, True, True), relabel(g.pins, False, True),
                        relabel(g.pinned, True, False), order)


def block_diagonal(graphs) -> CircuitGraph:
    """One graph whose relations are the block-diagonal stack of the given independent sub-graphs (cell and net
    ids of sub-graph q are shifted by the sizes of the sub-graphs before it).  A layer on this graph computes
    exactly what the layers on the sub-graphs compute, in one launch per kernel instead of one per sub-graph."""
    c_off = np.concatenate([[0], np.cumsum([g.Nc for g in graphs])]).astype(np.int64)
    n_off = np.concatenate([[0], np.cumsum([g.Nn for g in graphs])]).astype(np.int64)

    def stack(pats, col_off, n_cols):
        rp, ci, e = [np.zeros(1, np.int64)], [], 0
        for p, co in zip(pats, col_off):
            rp.append(p.rowptr[1:].astype(np.int64) + e)
            ci.append(p.colidx.astype(np.int64) + co)
            e += p.nnz
        assert e < 2 ** 31
        return Pattern(int(sum(p.n_rows for p in pats)), int(n_cols), np.concatenate(rp).astype(np.int32),
                       (np.concatenate(ci) if ci else np.zeros(0)).astype(np.int32))

    Nc, Nn = int(c_off[-1]), int(n_off[-1])
    return CircuitGraph(name="+".join(g.name for g in graphs), seed=graphs[0].seed, Nc=Nc, Nn=Nn,
                        near=stack([g.near for g in graphs], c_off, Nc), pins=stack([g.pins for g in graphs], c_off, Nc),
                        pinned=stack([g.pinned for g in graphs], n_off, Nn))


def make_graph(name: str, seed: int = 0, **override) -> CircuitGraph:
    """Build the three relation patterns of the named workload (see ``WORKLOADS``).
    Keyword overrides (e.g. ``Nc=..., Nn=..., grid=...``) derive scaled variants."""
    cfg = workload(name)
    cfg.update(override)
    Nc, Nn = int(cfg["Nc"]), int(cfg["Nn"])
    near = _make_near(Nc, tuple(cfg["grid"]), tuple(cfg["near_law"]), _rng(seed, _STREAM_NEAR))
    pins = _make_pins(Nn, Nc, float(cfg["net_mean"]), cfg["net_cap"], float(cfg["evil"]),
                      _rng(seed, _STREAM_NET_DEGREE), _rng(seed, _STREAM_NET_MEMBERS))
    pinned = transpose_pattern(pins)
    return CircuitGraph(name, seed, Nc, Nn, near, pins, pinned, placement_order(Nc, tuple(cfg["grid"])))


def make_tensors(Nc: int, Nn: int, D: int, seed: int = 0, upstream: bool = True) -> LayerTensors:
    """Features N(0,1), weights Xavier-uniform U(+-sqrt(6/(D+D))), upstream gradients N(0,1)."""
    X_cell = _rng(seed, _STREAM_X_CELL).standard_normal((Nc, D), dtype=np.float32)
    X_net = _rng(seed, _STREAM_X_NET).standard_normal((Nn, D), dtype=np.float32)
    bound = math.sqrt(6.0 / (D + D))
    rw = _rng(seed, _STREAM_WEIGHTS)
    W = {n: rw.uniform(-bound, bound, size=(D, D)).astype(np.float32) for n in WEIGHT_NAMES}
    t = LayerTensors(D=D, X_cell=X_cell, X_net=X_net, W=W)
    if upstream:
        ru = _rng(seed, _STREAM_UPSTREAM)
        t.dY_cell = ru.standard_normal((Nc, D), dtype=np.float32)
        t.dY_net = ru.standard_normal((Nn, D), dtype=np.float32)
    return t
