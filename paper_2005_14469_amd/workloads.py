"""Seeded synthetic inputs for the GCOO SpDM path.

This module only draws random matrices.  It holds none of the method's
arithmetic (no format conversion beyond assembling a CSR triple, no product),
so that the CPU oracle and the HIP path can both be fed from it without
sharing any code of the method itself.

The generators stand in for the uniformly random matrices of the paper's
evaluation (Section 4.2): square A with an exact number of nonzeros placed
uniformly at random, dense B.  A fifth, skewed workload (power-law row
lengths) stresses load balance.

Every generator uses ``numpy.random.default_rng(seed)`` (PCG64) and a fixed
draw order, so a (name, seed) pair names one input on every machine.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20051446


@dataclass
class Workload:
    """A = (row_ptr, col_idx, vals) in CSR (sorted columns), B dense row-major."""

    name: str
    m: int
    k: int
    N: int
    row_ptr: np.ndarray  # int32 [m+1]
    col_idx: np.ndarray  # int32 [nnz]
    vals: np.ndarray  # float32 [nnz]
    B: np.ndarray  # float32 [k, N]

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])


def csr_from_cells(m: int, k: int, cells: np.ndarray, vals: np.ndarray):
    """Assemble CSR from linear cell ids (row*k+col); columns sorted per row.

    ``vals[i]`` belongs to ``cells[i]``; both are reordered together.
    """
    order = np.argsort(cells, kind="stable")
    cells = cells[order]
    vals = np.ascontiguousarray(vals[order])
    rows = cells // k
    col_idx = (cells - rows * k).astype(np.int32)
    counts = np.bincount(rows, minlength=m)
    row_ptr = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    return row_ptr.astype(np.int32), col_idx, vals


def _draw(rng, dist: str, shape):
    if dist == "normal":
        return rng.standard_normal(shape, dtype=np.float32)
    if dist == "uniform":
        return (rng.random(shape, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)).astype(np.float32)
    raise ValueError(dist)


def uniform_random(m: int, k: int, N: int, sparsity: float, seed: int,
                   dist: str = "normal", name: str | None = None) -> Workload:
    """Exactly round((1-s)*m*k) nonzeros at cells drawn without replacement."""
    rng = np.random.default_rng(seed)
    nnz = int(round((1.0 - sparsity) * m * k))
    cells = rng.choice(m * k, size=nnz, replace=False)
    vals = _draw(rng, dist, nnz)
    B = _draw(rng, dist, (k, N))
    row_ptr, col_idx, vals = csr_from_cells(m, k, np.asarray(cells, dtype=np.int64), vals)
    return Workload(name or f"uniform_{m}x{k}_s{sparsity}", m, k, N, row_ptr, col_idx, vals, B)


def zipf_rows(m: int, k: int, N: int, seed: int, exponent: float = 1.5,
              row_max: int = 4096, name: str | None = None) -> Workload:
    """Row lengths ~ Zipf(exponent) redrawn until <= row_max; distinct uniform columns."""
    rng = np.random.default_rng(seed)
    lens = rng.zipf(exponent, size=m)
    bad = lens > row_max
    while bad.any():
        lens[bad] = rng.zipf(exponent, size=int(bad.sum()))
        bad = lens > row_max
    lens = np.minimum(lens, k).astype(np.int64)
    row_ptr = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(lens, out=row_ptr[1:])
    nnz = int(row_ptr[-1])
    col_idx = np.empty(nnz, dtype=np.int32)
    for i in range(m):
        L = int(lens[i])
        c = rng.choice(k, size=L, replace=False)
        c.sort()
        col_idx[row_ptr[i]:row_ptr[i + 1]] = c
    vals = _draw(rng, "normal", nnz)
    B = _draw(rng, "normal", (k, N))
    return Workload(name or f"zipf_{m}x{k}", m, k, N, row_ptr.astype(np.int32), col_idx, vals, B)


def diagonal(n: int, N: int, seed: int, name: str | None = None) -> Workload:
    """Diagonal A: the structure on which the paper's reuse search finds nothing (Section 4.1)."""
    rng = np.random.default_rng(seed)
    vals = _draw(rng, "normal", n)
    B = _draw(rng, "normal", (n, N))
    row_ptr = np.arange(n + 1, dtype=np.int32)
    col_idx = np.arange(n, dtype=np.int32)
    return Workload(name or f"diag_{n}", n, n, N, row_ptr, col_idx, vals, B)


# The five named configurations (index = position in the benchmark's config list).
CONFIGS = {
    0: dict(kind="uniform", m=256, k=256, N=256, sparsity=0.9, dist="normal"),
    1: dict(kind="uniform", m=4000, k=4000, N=4000, sparsity=0.95, dist="normal"),
    2: dict(kind="uniform", m=8000, k=8000, N=8000, sparsity=0.9, dist="normal"),
    3: dict(kind="uniform", m=8000, k=8000, N=8000, sparsity=0.995, dist="uniform"),
    4: dict(kind="zipf", m=16384, k=16384, N=512),
}


def config(index: int) -> Workload:
    c = CONFIGS[index]
    seed = BASE_SEED + index
    if c["kind"] == "uniform":
        return uniform_random(c["m"], c["k"], c["N"], c["sparsity"], seed, c["dist"],
                              name=f"config{index}_{c['m']}x{c['k']}_s{c['sparsity']}")
    return zipf_rows(c["m"], c["k"], c["N"], seed, name=f"config{index}_zipf_{c['m']}")
