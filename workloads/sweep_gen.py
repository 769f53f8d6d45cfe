"""Seeded population of synthetic matrices for training and evaluating the selector.

Stands in for the SuiteSparse collection the paper trains on (Sec. IV-B).  Matrix m
is square, rows = round(10^U(3,7)), and its row-length distribution is drawn from
five families:

  uniform  len ~ U{lo..hi}, lo ~ U{0..4}, hi = lo + round(10^U(0,2.5)); random columns
  banded   half bandwidth b = round(10^U(0,2)); row i holds columns [i-b, i+b] in range
  poisson  len ~ Poisson(10^U(0,1.8)); random columns
  zipf     len = min(Zipf(s), min(cols, 200000)), s ~ U(1.2, 2.5); random columns
  stencil  nearest-neighbour stencil on a regular grid, natural ordering: 5 points on an
           n x n grid or 7 points on an n x n x n grid (n from the row count), boundary
           rows shorter; the structure of discretised PDEs, which the collection the
           paper trains on is full of and which no random-column family resembles

If nnz exceeds the cap (2e8 by default) the row count is halved until it fits.
Shape parameters and row lengths come from numpy (PCG64, seed 170175 + 1000 m) on the
host; the bulk arrays (columns, values, x) are drawn with torch on the chosen device
from a generator seeded with the same number, so a population can be produced on the
GPU in seconds.  (A torch CPU generator and a GPU generator give different streams:
a matrix is reproducible per device type.)  Holds no SpMV / feature arithmetic.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

FAMILIES = ("uniform", "banded", "poisson", "zipf", "stencil")
SWEEP_SEED = 170170 + 5


@dataclass
class SweepSpec:
    m: int
    family: str
    rows: int
    params: dict
    lens: np.ndarray  # int64 [rows]

    @property
    def nnz(self) -> int:
        return int(self.lens.sum())


def sweep_spec(m: int, nnz_cap: int = 200_000_000, max_rows_exp: float = 7.0) -> SweepSpec:
    rng = np.random.default_rng(SWEEP_SEED + 1000 * m)
    rows = int(round(10 ** rng.uniform(3.0, max_rows_exp)))
    family = FAMILIES[int(rng.integers(len(FAMILIES)))]
    params: dict = {}
    if family == "uniform":
        lo = int(rng.integers(0, 5))
        hi = lo + int(round(10 ** rng.uniform(0.0, 2.5)))
        params = {"lo": lo, "hi": hi}
        lens = rng.integers(lo, hi + 1, rows)
    elif family == "banded":
        b = int(round(10 ** rng.uniform(0.0, 2.0)))
        params = {"b": b}
        i = np.arange(rows, dtype=np.int64)
        lens = np.minimum(i + b, rows - 1) - np.maximum(i - b, 0) + 1
    elif family == "stencil":
        dim = int(rng.integers(2, 4))
        n = max(2, int(round(rows ** (1.0 / dim))))
        rows = n ** dim
        params = {"dim": dim, "n": n}
        lens = stencil_mask_numpy(n, dim).sum(axis=1)
    elif family == "poisson":
        lam = float(10 ** rng.uniform(0.0, 1.8))
        params = {"lam": lam}
        lens = rng.poisson(lam, rows)
    else:
        s = float(rng.uniform(1.2, 2.5))
        params = {"s": s}
        lens = np.minimum(rng.zipf(s, rows), min(rows, 200_000))
    lens = np.minimum(np.asarray(lens, dtype=np.int64), rows)
    while int(lens.sum()) > nnz_cap and rows > 1:
        rows //= 2
        if family == "banded":   # the band is clipped by the new last row
            i = np.arange(rows, dtype=np.int64)
            lens = np.minimum(i + params["b"], rows - 1) - np.maximum(i - params["b"], 0) + 1
        else:
            lens = np.minimum(lens[:rows], rows)
    return SweepSpec(m, family, rows, params, lens)


def stencil_offsets(n: int, dim: int):
    """Column offsets of the stencil, ascending: -n^(dim-1) .. -n, -1, 0, +1, +n .. ."""
    strides = [n ** d for d in range(dim)]            # x is the fastest coordinate
    return [-st for st in reversed(strides)] + [0] + strides


def stencil_mask_numpy(n: int, dim: int) -> np.ndarray:
    """[rows, 2 dim + 1] bool: which stencil points of each grid point lie inside the grid."""
    rows = n ** dim
    i = np.arange(rows, dtype=np.int64)
    coord = [(i // n ** d) % n for d in range(dim)]   # coord[0] = x
    lower = [coord[d] > 0 for d in reversed(range(dim))]
    upper = [coord[d] < n - 1 for d in range(dim)]
    return np.stack(lower + [np.ones(rows, bool)] + upper, axis=1)


def build_on_device(spec: SweepSpec, device="cuda:0"):
    """Returns (row_ptr int32, col_idx int32, values fp32, x fp32) as torch tensors on
    `device`; columns ascending inside each row."""
    import torch
    rows, cols = spec.rows, spec.rows
    gen = torch.Generator(device=device)
    gen.manual_seed(SWEEP_SEED + 1000 * spec.m)
    rp64 = np.zeros(rows + 1, dtype=np.int64)
    np.cumsum(spec.lens, out=rp64[1:])
    nnz = int(rp64[-1])
    assert nnz < 2**31
    row_ptr = torch.from_numpy(rp64.astype(np.int32)).to(device)
    lens_d = torch.from_numpy(spec.lens).to(device)
    row_id = torch.repeat_interleave(torch.arange(rows, device=device, dtype=torch.int64), lens_d,
                                     output_size=nnz)
    if spec.family == "stencil":
        n, dim = spec.params["n"], spec.params["dim"]
        i = torch.arange(rows, device=device, dtype=torch.int64)
        coord = [(i // n ** d) % n for d in range(dim)]
        mask = torch.stack([coord[d] > 0 for d in reversed(range(dim))] + [torch.ones_like(i, dtype=torch.bool)]
                           + [coord[d] < n - 1 for d in range(dim)], dim=1)
        offs = torch.tensor(stencil_offsets(n, dim), device=device, dtype=torch.int64)
        col = (i[:, None] + offs[None, :])[mask]          # row-major: rows in order, ascending inside a row
        del mask, coord, i
    elif spec.family == "banded":
        b = spec.params["b"]
        first = torch.clamp(torch.arange(rows, device=device, dtype=torch.int64) - b, min=0)
        start = torch.from_numpy(rp64[:-1]).to(device)
        col = torch.arange(nnz, device=device, dtype=torch.int64) - start[row_id] + first[row_id]
    else:
        col = torch.randint(0, cols, (nnz,), generator=gen, device=device, dtype=torch.int64)
        key, _ = torch.sort(row_id * cols + col)
        col = key - row_id * cols
        del key
    col_idx = col.to(torch.int32)
    del col, row_id
    values = torch.rand(nnz, generator=gen, device=device, dtype=torch.float32) * 2 - 1
    x = torch.rand(cols, generator=gen, device=device, dtype=torch.float32) * 2 - 1
    return row_ptr, col_idx, values, x
