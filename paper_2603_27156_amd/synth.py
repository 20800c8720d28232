"""Seeded synthetic inputs for the GSR-GNN training-step path.

This module only draws random numbers and lays them out as arrays: a directed
circuit-like DAG in CSR form, node features, regression targets and weight
initialisations.  It holds none of the method's arithmetic (no normalisation, no
top-k, no message passing), so the CPU oracle and the HIP library can both be fed
from it without sharing any code of the method itself.

The graphs stand in for the sampled CircuitNet designs the paper trains on
(Section 5, "Dataset"; Table 1), which are not available here.  They follow the
paper's description of circuit graphs (Section 2, Figure 5): locally regular
connectivity plus a few very-high-fanout nets.

Draw order for one configuration (never reordered, so seeds stay meaningful):
graph -> X0 -> targets -> W (layer-major, group-minor) -> w_out.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional, Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class GsrWorkload:
    """Shape of one workload (names follow the paper: N, D, C, L, k)."""

    name: str
    n: int                      # nodes N
    levels: int                 # topological levels of the DAG
    fanin_p: Tuple[float, ...]  # P(fan-in = 1, 2, ...)
    alpha: Optional[float]      # power-law exponent of the source choice (None: uniform)
    hubs: int                   # number of global high-fanout nets (level 0)
    hub_degree: int             # fan-out of each global net
    d: int                      # feature width D
    c: int                      # groups C
    l: int                      # layers L
    k: int                      # retained elements per row per group
    norm: str                   # "none" | "rms"
    dtype: str                  # "f32" | "bf16"
    rowptr64: bool = False      # row pointers handed over as int64

    @property
    def dg(self) -> int:
        return self.d // self.c


WORKLOADS = {
    0: GsrWorkload("cfg0-tiny-2k", 2_000, 20, (0.3, 0.5, 0.2), None, 0, 0,
                   64, 2, 4, 8, "none", "f32"),
    1: GsrWorkload("cfg1-100k", 100_000, 200, (0.3, 0.5, 0.2), 1.2, 0, 0,
                   128, 2, 28, 16, "rms", "f32"),
    2: GsrWorkload("cfg2-1M", 1_000_000, 1_000, (0.25, 0.25, 0.25, 0.25), 1.2, 8, 5_000,
                   256, 4, 112, 16, "rms", "f32"),
    # cfg3 is cfg2's graph at other depths; use workload(3, l=...)
    3: GsrWorkload("cfg3-1M-depth", 1_000_000, 1_000, (0.25, 0.25, 0.25, 0.25), 1.2, 8, 5_000,
                   256, 4, 448, 16, "rms", "f32"),
    4: GsrWorkload("cfg4-8M", 8_000_000, 4_000, (0.25, 0.25, 0.25, 0.25), 1.1, 8, 50_000,
                   256, 8, 112, 8, "rms", "bf16", True),
    # Shaped like the graphs of the paper's Table 1 / Table 2 (about 50k nodes, 12M edges: mean degree
    # about 246; 100 layers, 384 channels): the regime where the neighbour gather dominates.  Used for
    # the sweep over k.  384 channels as 6 groups of 64 (the paper runs C = 2).
    5: GsrWorkload("dense-50k", 49_600, 50, tuple([1.0 / 245.0] * 245), None, 0, 0,
                   384, 6, 100, 16, "rms", "f32"),
}


def workload(i: int, **overrides) -> GsrWorkload:
    w = WORKLOADS[i]
    return replace(w, **overrides) if overrides else w


def scaled(w: GsrWorkload, n: int, levels: Optional[int] = None, **overrides) -> GsrWorkload:
    """Same recipe at another node count (used for parity cases the oracle finishes quickly)."""
    lv = levels if levels is not None else max(4, int(round(w.levels * n / w.n)))
    lv = max(1, min(lv, n))
    hub_deg = min(w.hub_degree, max(0, n // 4))
    return replace(w, n=n, levels=lv, hub_degree=hub_deg, **overrides)


def _level_bounds(n: int, levels: int) -> np.ndarray:
    """First node id of every level (level-major numbering), length levels+1."""
    return (np.arange(levels + 1, dtype=np.int64) * n) // levels


def circuit_dag(w: GsrWorkload, rng: np.random.Generator):
    """Directed level/fan-in DAG as CSR (row = sink node, columns = its fan-in sources).

    Every node of level >= 1 draws a fan-in q from `fanin_p` and then q sources, with
    replacement, from the window made of the previous (up to) three levels; the source is
    uniform, or has probability proportional to (rank+1)^-alpha where rank is its position
    in the window in ascending node id.  Duplicate draws are merged.  `hubs` level-0 nodes
    are additionally wired to `hub_degree` distinct later nodes each (clock/reset-like nets).
    Returns (rowptr int64 [n+1], colidx int32 [nnz]) with ascending columns per row.
    """
    n, levels = w.n, w.levels
    lb = _level_bounds(n, levels)
    level_of = np.searchsorted(lb, np.arange(n, dtype=np.int64), side="right") - 1
    qmax = len(w.fanin_p)
    q = rng.choice(np.arange(1, qmax + 1), size=n, p=np.asarray(w.fanin_p, dtype=np.float64))
    q[level_of == 0] = 0
    u = rng.random((n, qmax))                      # one uniform per potential source slot
    lo = lb[np.maximum(level_of - 3, 0)]
    hi = lb[level_of]
    width = (hi - lo).astype(np.int64)             # window size; 0 only on level 0
    src = np.full((n, qmax), -1, dtype=np.int64)
    if w.alpha is None:
        r = np.minimum((u * width[:, None]).astype(np.int64), np.maximum(width[:, None] - 1, 0))
    else:
        r = np.zeros((n, qmax), dtype=np.int64)
        for wd in np.unique(width):
            if wd == 0:
                continue
            rows = np.nonzero(width == wd)[0]
            pmf = (np.arange(1, wd + 1, dtype=np.float64)) ** (-w.alpha)
            cdf = np.cumsum(pmf)
            cdf /= cdf[-1]
            rr = np.searchsorted(cdf, u[rows], side="right")
            r[rows] = np.minimum(rr, wd - 1)
    slot = np.arange(qmax)[None, :]
    valid = slot < q[:, None]
    src = np.where(valid, lo[:, None] + r, -1)
    rows = np.repeat(np.arange(n, dtype=np.int64), qmax)[valid.ravel()]
    cols = src.ravel()[valid.ravel()]
    if w.hubs > 0 and w.hub_degree > 0:
        first_late = int(lb[1])
        for h in range(w.hubs):
            sinks = rng.choice(np.arange(first_late, n, dtype=np.int64), size=min(w.hub_degree, n - first_late),
                               replace=False)
            rows = np.concatenate([rows, sinks])
            cols = np.concatenate([cols, np.full(sinks.shape, h, dtype=np.int64)])
    key = np.unique(rows * np.int64(n) + cols)      # merge duplicates, sort by (row, col)
    rows = key // n
    cols = (key % n).astype(np.int32)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rowptr, rows + 1, 1)
    rowptr = np.cumsum(rowptr)
    return rowptr, cols


def glorot_uniform(rng: np.random.Generator, fan_in: int, fan_out: int, shape) -> np.ndarray:
    a = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-a, a, size=shape).astype(np.float32)


@dataclass
class GsrInputs:
    w: GsrWorkload
    rowptr: np.ndarray      # int64 (or int32 when not rowptr64) [n+1], directed input graph
    colidx: np.ndarray      # int32 [nnz]
    x0: np.ndarray          # float32 [n, d]
    target: np.ndarray      # float32 [n]
    weights: np.ndarray     # float32 [l, c, dg, dg]  (in -> out)
    w_out: np.ndarray       # float32 [d]
    b_out: float = 0.0


def make_inputs(w: GsrWorkload, seed: int = 0, l_weights: Optional[int] = None) -> GsrInputs:
    """All arrays of one workload.  `l_weights` draws weights for a deeper stack than w.l
    (depth sweeps reuse prefixes of one draw)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    rowptr, colidx = circuit_dag(w, rng)
    if not w.rowptr64:
        rowptr = rowptr.astype(np.int32)
    x0 = rng.standard_normal((w.n, w.d), dtype=np.float32)
    target = rng.standard_normal(w.n, dtype=np.float32)
    lw = l_weights if l_weights is not None else w.l
    weights = glorot_uniform(rng, w.dg, w.dg, (lw, w.c, w.dg, w.dg))
    w_out = glorot_uniform(rng, w.d, 1, (w.d,))
    return GsrInputs(w, rowptr, colidx, x0, target, weights, w_out, 0.0)


def to_bf16_grid(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even) and return them as float32.
    Pure bit manipulation of the input format; used to prepare inputs of the bf16-storage runs."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)
