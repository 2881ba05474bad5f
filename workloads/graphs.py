"""Seeded generators for the five benchmark configurations.

Each configuration is a synthetic stand-in with the node count, degree
distribution, value normalisation and feature shape of one of the paper's
workloads (dataset statistics table: Pubmed / Arxiv / Proteins / Reddit); no
dataset is reproduced, only its shape.  Everything is vectorised NumPy driven
by ``numpy.random.default_rng(seed)`` so a (config, scale) pair always yields
the same arrays.

CSR conventions used everywhere in this repository:
  * ``rowptr`` int32 [N+1], ``rowptr[0] == 0``, non-decreasing;
  * ``colidx`` int32 [nnz], strictly increasing inside a row (so "the first W
    entries of a row" means its W lowest-numbered neighbours);
  * ``vals``   float32 [nnz];
  * every row holds its own self-loop.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

CONFIG_IDS = (1, 2, 3, 4, 5)

_STRUCT_SEED = 1000   # + config id : graph structure
_FEAT_SEED = 2000     # + config id : feature matrix
_WEIGHT_SEED = 3000   # + config id : dense layer weights (config 5)


@dataclass
class Workload:
    cfg: int
    name: str
    rowptr: np.ndarray
    colidx: np.ndarray
    vals: np.ndarray
    X: np.ndarray            # [N, ldx] float32, columns >= F are zero padding
    F: int
    Ws: Tuple[int, ...]      # sampling widths the configuration sweeps
    extras: Dict[str, np.ndarray] = field(default_factory=dict)

    @property
    def N(self) -> int:
        return int(self.rowptr.shape[0] - 1)

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    @property
    def ldx(self) -> int:
        return int(self.X.shape[1])

    @property
    def max_degree(self) -> int:
        return int(np.diff(self.rowptr).max()) if self.N else 0


# --------------------------------------------------------------------------
# structure helpers
# --------------------------------------------------------------------------
def powerlaw_degrees(n: int, mean: float, dmax: int, rng: np.random.Generator,
                     exponent: float = 2.1) -> np.ndarray:
    """Degrees with density ~ d**-exponent on [dmin, dmax], dmin calibrated by
    bisection (on one fixed set of uniform draws) so the sample mean is `mean`."""
    u = rng.random(n)
    tail = -1.0 / (exponent - 1.0)
    shape = u ** tail                      # Pareto(1) multiples, >= 1

    def realised(dmin: float) -> np.ndarray:
        return np.clip(np.floor(dmin * shape), 1, dmax)

    lo, hi = 0.05, float(dmax)
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if realised(mid).mean() < mean:
            lo = mid
        else:
            hi = mid
    return realised(hi).astype(np.int64)


def csr_from_pairs(n: int, rows: np.ndarray, cols: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Sort (row, col) pairs, drop duplicates, return int32 (rowptr, colidx)."""
    key = (rows.astype(np.int64) << np.int64(32)) | cols.astype(np.int64)
    key.sort()
    if key.size:
        keep = np.empty(key.shape, dtype=bool)
        keep[0] = True
        np.not_equal(key[1:], key[:-1], out=keep[1:])
        key = key[keep]
    r = key >> np.int64(32)
    c = (key & np.int64(0xFFFFFFFF)).astype(np.int32)
    counts = np.bincount(r, minlength=n)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    assert rowptr[-1] < 2 ** 31, "nnz must fit int32"
    return rowptr.astype(np.int32), c


def csr_from_degrees(n: int, deg: np.ndarray, rng: np.random.Generator,
                     blocks: int = 0, p_intra: float = 0.0) -> Tuple[np.ndarray, np.ndarray]:
    """Row i gets deg[i] random targets (uniform, or clustered: with probability
    `p_intra` inside the row's own block of `n/blocks` contiguous ids) plus a
    self-loop; duplicates collapse."""
    total = int(deg.sum())
    rows = np.repeat(np.arange(n, dtype=np.int64), deg)
    cols = rng.integers(0, n, size=total, dtype=np.int64)
    if blocks > 1:
        bsize = -(-n // blocks)
        intra = rng.random(total) < p_intra
        start = (rows // bsize) * bsize
        width = np.minimum(start + bsize, n) - start
        local = start + (rng.random(total) * width).astype(np.int64)
        cols = np.where(intra, local, cols)
        del intra, start, width, local
    loops = np.arange(n, dtype=np.int64)
    rows = np.concatenate([rows, loops])
    cols = np.concatenate([cols, loops])
    return csr_from_pairs(n, rows, cols)


def random_csr(n: int, avg_deg: float, seed: int, self_loops: bool = True,
               empty_frac: float = 0.0) -> Tuple[np.ndarray, np.ndarray]:
    """Small unstructured test graph: Poisson degrees, optional empty rows."""
    rng = np.random.default_rng(seed)
    deg = rng.poisson(avg_deg, size=n).astype(np.int64)
    deg = np.minimum(deg, n)
    empty = rng.random(n) < empty_frac
    deg[empty] = 0
    rows = np.repeat(np.arange(n, dtype=np.int64), deg)
    cols = rng.integers(0, n, size=int(deg.sum()), dtype=np.int64)
    if self_loops:
        loops = np.arange(n, dtype=np.int64)[~empty]
        rows = np.concatenate([rows, loops])
        cols = np.concatenate([cols, loops])
    return csr_from_pairs(n, rows, cols)


def _row_lengths(rowptr: np.ndarray) -> np.ndarray:
    return np.diff(rowptr.astype(np.int64))


def sym_norm_vals(rowptr: np.ndarray, colidx: np.ndarray) -> np.ndarray:
    """a_ij = 1/sqrt(d_i d_j), d = CSR row length (self-loop included)."""
    d = _row_lengths(rowptr).astype(np.float64)
    inv = np.zeros_like(d)
    np.divide(1.0, np.sqrt(d), out=inv, where=d > 0)
    rows_inv = np.repeat(inv, _row_lengths(rowptr))
    return (rows_inv * inv[colidx]).astype(np.float32)


def mean_agg_vals(rowptr: np.ndarray) -> np.ndarray:
    """a_ij = 1/d_i."""
    d = _row_lengths(rowptr)
    inv = np.zeros(d.shape, dtype=np.float64)
    np.divide(1.0, d, out=inv, where=d > 0)
    return np.repeat(inv, d).astype(np.float32)


def _uniform_pm1(rng: np.random.Generator, shape) -> np.ndarray:
    x = rng.random(shape, dtype=np.float32)
    x *= 2.0
    x -= 1.0
    return x


def _glorot(rng: np.random.Generator, fan_in: int, fan_out: int) -> np.ndarray:
    lim = np.sqrt(6.0 / (fan_in + fan_out))
    return (_uniform_pm1(rng, (fan_in, fan_out)) * np.float32(lim)).astype(np.float32)


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------
def _scaled(n: int, scale: float, floor: int = 64) -> int:
    return max(floor, int(round(n * scale)))


def _cfg1(scale: float) -> Workload:
    n = _scaled(2708, scale)
    rng = np.random.default_rng(_STRUCT_SEED + 1)
    m = 2 * n
    a = rng.integers(0, n, size=m, dtype=np.int64)
    b = rng.integers(0, n, size=m, dtype=np.int64)
    loops = np.arange(n, dtype=np.int64)
    rows = np.concatenate([a, b, loops])
    cols = np.concatenate([b, a, loops])
    rowptr, colidx = csr_from_pairs(n, rows, cols)
    vals = sym_norm_vals(rowptr, colidx)
    X = _uniform_pm1(np.random.default_rng(_FEAT_SEED + 1), (n, 16))
    maxdeg = int(np.diff(rowptr).max())
    return Workload(1, "tiny-gcn", rowptr, colidx, vals, X, 16, (4, 8, maxdeg))


def _cfg2(scale: float) -> Workload:
    n = _scaled(170_000, scale)
    rng = np.random.default_rng(_STRUCT_SEED + 2)
    deg = powerlaw_degrees(n, 14.0 - 1.0, min(13_000, n // 2), rng)   # +1 self-loop
    rowptr, colidx = csr_from_degrees(n, deg, rng)
    vals = sym_norm_vals(rowptr, colidx)
    X = np.random.default_rng(_FEAT_SEED + 2).standard_normal((n, 128), dtype=np.float32)
    return Workload(2, "citation-like", rowptr, colidx, vals, X, 128, (16, 32, 64, 128))


def _cfg3_graph(scale: float):
    n = _scaled(233_000, scale)
    rng = np.random.default_rng(_STRUCT_SEED + 3)
    mean = 490.0 if scale >= 1.0 else max(8.0, 490.0 * min(1.0, scale * 8))
    deg = powerlaw_degrees(n, mean, min(21_000, n // 4), rng)
    rowptr, colidx = csr_from_degrees(n, deg, rng)
    return n, rowptr, colidx


def _cfg3(scale: float) -> Workload:
    n, rowptr, colidx = _cfg3_graph(scale)
    vals = mean_agg_vals(rowptr)
    X = _uniform_pm1(np.random.default_rng(_FEAT_SEED + 3), (n, 64))
    return Workload(3, "social-like", rowptr, colidx, vals, X, 64, (16, 32, 64, 128, 256))


def _cfg4(scale: float) -> Workload:
    n = _scaled(2_450_000, scale)
    rng = np.random.default_rng(_STRUCT_SEED + 4)
    deg = powerlaw_degrees(n, 50.0 - 1.0, min(20_000, n // 4), rng)
    rowptr, colidx = csr_from_degrees(n, deg, rng, blocks=64, p_intra=0.8)
    vals = sym_norm_vals(rowptr, colidx)
    X = np.zeros((n, 128), dtype=np.float32)
    X[:, :100] = np.random.default_rng(_FEAT_SEED + 4).standard_normal((n, 100), dtype=np.float32)
    # F = 128: the zero padding is part of the matrix the kernel multiplies.
    return Workload(4, "copurchase-like", rowptr, colidx, vals, X, 128, (32, 64, 128))


def gcn_operands(n: int):
    """Dense operands of config 5 for an n-node graph: X0 [n x 602] uniform[-1,1],
    W1 [602 x 256] and W2 [256 x 41] Glorot-uniform."""
    X0 = _uniform_pm1(np.random.default_rng(_FEAT_SEED + 5), (n, 602))
    wrng = np.random.default_rng(_WEIGHT_SEED + 5)
    W1 = _glorot(wrng, 602, 256)
    W2 = _glorot(wrng, 256, 41)
    return X0, W1, W2


def _cfg5(scale: float) -> Workload:
    """Config-3 graph plus the dense operands of a 2-layer GCN forward.  `X` is
    the first layer's input X0 [N x 602]; `extras` holds W1 [602 x 256] and
    W2 [256 x 41].  The SpMM stages run on X0*W1 (F=256) and on
    relu(.)*W2 (F=41); the caller forms those products."""
    n, rowptr, colidx = _cfg3_graph(scale)
    vals = mean_agg_vals(rowptr)
    X0, W1, W2 = gcn_operands(n)
    return Workload(5, "gcn2-feature-sweep", rowptr, colidx, vals, X0, 602, (64,),
                    extras={"W1": W1, "W2": W2})


_BUILDERS = {1: _cfg1, 2: _cfg2, 3: _cfg3, 4: _cfg4, 5: _cfg5}


def make_workload(cfg: int, scale: float = 1.0) -> Workload:
    """Build configuration `cfg` (1..5).  `scale` < 1 shrinks the node count
    (and, for the dense graph, the mean degree) for CPU-sized test cases while
    keeping the recipe; `scale == 1` is the benchmark size."""
    if cfg not in _BUILDERS:
        raise ValueError(f"unknown config {cfg}")
    return _BUILDERS[cfg](float(scale))
