"""Seeded synthetic CSR matrices shaped like the SpMV workloads of the Seer case study.

The case study (Sec. IV-B) measures on the SuiteSparse collection, which is not
available offline; these generators stand in for it.  They hold no SpMV, feature
or selector arithmetic: they only draw structure (row lengths, column indices)
and values.  Both the CPU oracle's tests and the HIP path's tests take their
inputs from here, so the two sides see byte-identical arrays.

Conventions shared by every generator:
  * int32 ``row_ptr`` / ``col_idx``, float32 ``values``; ``row_ptr[0] == 0``;
  * column indices ascending inside a row; where columns are drawn with
    replacement, repeated columns are kept (an SpMV sums them);
  * values and the dense vector ``x`` are uniform in [-1, 1);
  * all randomness comes from ``numpy.random.default_rng(seed)`` (PCG64) and is
    consumed in a fixed order, bulk draws in blocks of ``_BLOCK`` nonzeros, so a
    seed names one matrix on every machine.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 170170
_BLOCK = 1 << 25  # nonzeros drawn per bulk call; part of the recipe


@dataclass
class HostCSR:
    rows: int
    cols: int
    row_ptr: np.ndarray  # int32 [rows + 1]
    col_idx: np.ndarray  # int32 [nnz]
    values: np.ndarray   # float32 [nnz]
    name: str = ""

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1]) if self.row_ptr.size else 0

    def validate(self) -> None:
        rp, ci = self.row_ptr, self.col_idx
        assert rp.dtype == np.int32 and ci.dtype == np.int32 and self.values.dtype == np.float32
        assert rp.shape == (self.rows + 1,) and rp[0] == 0
        assert np.all(np.diff(rp.astype(np.int64)) >= 0)
        assert ci.shape == (self.nnz,) and self.values.shape == (self.nnz,)
        if self.nnz:
            assert ci.min() >= 0 and ci.max() < self.cols


def config_seed(config_number: int) -> int:
    return BASE_SEED + config_number


def dense_vector(n: int, seed: int) -> np.ndarray:
    """x uniform in [-1, 1), float32, drawn from its own stream (seed + 7919)."""
    rng = np.random.default_rng(seed + 7919)
    return rng.uniform(-1.0, 1.0, n).astype(np.float32)


def _row_ptr_from_lengths(lens: np.ndarray) -> np.ndarray:
    total = int(lens.sum(dtype=np.int64))
    if total >= 2**31:
        raise ValueError(f"nnz {total} does not fit int32")
    rp = np.zeros(lens.size + 1, dtype=np.int64)
    np.cumsum(lens, out=rp[1:])
    return rp.astype(np.int32)


def _uniform_values(rng: np.random.Generator, nnz: int) -> np.ndarray:
    out = np.empty(nnz, dtype=np.float32)
    for a in range(0, nnz, _BLOCK):
        b = min(a + _BLOCK, nnz)
        out[a:b] = rng.uniform(-1.0, 1.0, b - a)
    return out


def _sorted_random_columns(rng: np.random.Generator, row_ptr: np.ndarray, cols: int) -> np.ndarray:
    """Uniform columns with replacement, ascending inside each row.

    Rows are taken in blocks holding at most ``_BLOCK`` nonzeros (a single longer
    row forms a block of its own); inside a block the pairs (row, column) are
    sorted as one composite integer key.
    """
    rows = row_ptr.size - 1
    nnz = int(row_ptr[-1])
    out = np.empty(nnz, dtype=np.int32)
    r0 = 0
    rp64 = row_ptr.astype(np.int64)
    while r0 < rows:
        # furthest r1 with rp[r1] - rp[r0] <= _BLOCK, at least one row
        r1 = int(np.searchsorted(rp64, rp64[r0] + _BLOCK, side="right")) - 1
        r1 = min(max(r1, r0 + 1), rows)
        a, b = int(rp64[r0]), int(rp64[r1])
        if b > a:
            c = rng.integers(0, cols, b - a, dtype=np.int64)
            rid = np.repeat(np.arange(r1 - r0, dtype=np.int64), np.diff(rp64[r0:r1 + 1]))
            key = rid * cols + c
            key.sort()
            out[a:b] = key - rid * cols
        r0 = r1
    return out


def from_row_lengths(lens: np.ndarray, cols: int, rng: np.random.Generator, name: str = "") -> HostCSR:
    lens = np.asarray(lens, dtype=np.int64)
    rp = _row_ptr_from_lengths(lens)
    ci = _sorted_random_columns(rng, rp, cols)
    va = _uniform_values(rng, int(rp[-1]))
    return HostCSR(lens.size, cols, rp, ci, va, name)


# --------------------------------------------------------------------------
# Config 1: exactly k distinct uniformly random columns per row.
# --------------------------------------------------------------------------
def fixed_degree(rows: int = 4096, cols: int = 4096, k: int = 16, seed: int | None = None) -> HostCSR:
    seed = config_seed(1) if seed is None else seed
    rng = np.random.default_rng(seed)
    if k > cols:
        raise ValueError("k > cols")
    ci = np.empty((rows, k), dtype=np.int32)
    for r in range(rows):
        ci[r] = np.sort(rng.choice(cols, size=k, replace=False))
    rp = (np.arange(rows + 1, dtype=np.int64) * k).astype(np.int32)
    va = _uniform_values(rng, rows * k)
    return HostCSR(rows, cols, rp, ci.reshape(-1), va, f"fixed{k}_{rows}x{cols}")


# --------------------------------------------------------------------------
# Config 2: 5-point Laplacian on an n x n grid, natural row-major ordering,
# Dirichlet boundary (neighbours outside the grid are dropped).
# --------------------------------------------------------------------------
def laplacian_5pt(n: int = 1024) -> HostCSR:
    N = n * n
    idx = np.arange(N, dtype=np.int64)
    r, c = idx // n, idx % n
    # candidate columns in ascending order: up, left, centre, right, down
    cand = np.stack([idx - n, idx - 1, idx, idx + 1, idx + n], axis=1)
    keep = np.stack([r > 0, c > 0, np.ones(N, bool), c < n - 1, r < n - 1], axis=1)
    vals = np.broadcast_to(np.array([-1, -1, 4, -1, -1], dtype=np.float32), (N, 5))
    lens = keep.sum(axis=1)
    rp = _row_ptr_from_lengths(lens)
    return HostCSR(N, N, rp, cand[keep].astype(np.int32), np.ascontiguousarray(vals[keep]),
                   f"laplace5_{n}x{n}")


# --------------------------------------------------------------------------
# Config 3: power-law rows.  len = min(Zipf(s), cap).
# --------------------------------------------------------------------------
def zipf_rows(rows: int = 2_000_000, cols: int | None = None, s: float = 1.6,
              cap: int = 200_000, seed: int | None = None) -> HostCSR:
    seed = config_seed(3) if seed is None else seed
    cols = rows if cols is None else cols
    rng = np.random.default_rng(seed)
    lens = np.minimum(rng.zipf(s, rows), min(cap, cols))
    return from_row_lengths(lens, cols, rng, f"zipf{s}_{rows}")


# --------------------------------------------------------------------------
# Config 4: a fixed fraction of empty rows, the rest zero-truncated Poisson.
# --------------------------------------------------------------------------
def empty_poisson(rows: int = 8_000_000, cols: int = 1_000_000, empty_frac: float = 0.3,
                  lam: float = 4.0, seed: int | None = None) -> HostCSR:
    seed = config_seed(4) if seed is None else seed
    rng = np.random.default_rng(seed)
    n_empty = int(round(rows * empty_frac))
    perm = rng.permutation(rows)
    lens = np.zeros(rows, dtype=np.int64)
    live = perm[n_empty:]
    draw = rng.poisson(lam, live.size)
    while True:
        z = np.flatnonzero(draw == 0)
        if z.size == 0:
            break
        draw[z] = rng.poisson(lam, z.size)
    lens[live] = draw
    return from_row_lengths(lens, cols, rng, f"empty{empty_frac}_poisson{lam}_{rows}x{cols}")


# --------------------------------------------------------------------------
# Extra shapes used by tests (not BASELINE configs).
# --------------------------------------------------------------------------
def banded(rows: int, half_bandwidth: int, seed: int) -> HostCSR:
    """Square; row i holds every column in [i-b, i+b] that exists."""
    rng = np.random.default_rng(seed)
    i = np.arange(rows, dtype=np.int64)
    lo = np.maximum(i - half_bandwidth, 0)
    hi = np.minimum(i + half_bandwidth, rows - 1)
    lens = hi - lo + 1
    rp = _row_ptr_from_lengths(lens)
    nnz = int(rp[-1])
    rid = np.repeat(i, lens)
    ci = (np.arange(nnz, dtype=np.int64) - rp[:-1].astype(np.int64)[rid] + lo[rid]).astype(np.int32)
    return HostCSR(rows, rows, rp, ci, _uniform_values(rng, nnz), f"band{half_bandwidth}_{rows}")


def random_lengths(rows: int, cols: int, lo: int, hi: int, seed: int) -> HostCSR:
    """Row lengths uniform on {lo..hi} (clipped to cols)."""
    rng = np.random.default_rng(seed)
    lens = np.minimum(rng.integers(lo, hi + 1, rows), cols)
    return from_row_lengths(lens, cols, rng, f"unif{lo}-{hi}_{rows}x{cols}")


def explicit_lengths(lens, cols: int, seed: int, name: str = "explicit") -> HostCSR:
    """Caller fixes every row length (edge-case matrices in the tests)."""
    rng = np.random.default_rng(seed)
    return from_row_lengths(np.asarray(lens, dtype=np.int64), cols, rng, name)


def small_integer_values(A: HostCSR, seed: int, lo: int = -4, hi: int = 4) -> HostCSR:
    """Same structure, values replaced by small integers (sums exact in fp32)."""
    rng = np.random.default_rng(seed)
    v = rng.integers(lo, hi + 1, A.nnz).astype(np.float32)
    return HostCSR(A.rows, A.cols, A.row_ptr, A.col_idx, v, A.name + "_intvals")


def int32_limit(rows: int = 2_097_155, cols: int = 1 << 20, long_row: int = 5_000_000,
                seed: int = BASE_SEED + 31) -> HostCSR:
    """The largest matrix int32 offsets can express: exactly 2^31 - 1 nonzeros (16 GiB of
    entries).  Row lengths: uniform on 0..2047, every tenth row emptied, one row of
    ``long_row`` entries in the middle, all scaled down and topped up one by one to hit the
    total.  One block of ``_BLOCK`` columns (uniform, NOT ascending inside a row, unlike the
    other generators) and integer values in [-8, 7] is drawn and laid down 64 times, the
    columns shifted by 9973 per repetition (mod ``cols``) and the values rotated by 977
    entries per repetition, so that a matrix of this size is made in seconds."""
    target = (1 << 31) - 1
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, 2048, rows).astype(np.int64)
    lens[::10] = 0
    lens[rows // 2] = long_row
    lens = lens * target // int(lens.sum())
    short = target - int(lens.sum())                  # < rows: lost to the roundings
    assert 0 <= short < rows
    lens[np.flatnonzero(lens > 0)[:short]] += 1
    row_ptr = _row_ptr_from_lengths(lens)
    assert int(row_ptr[-1]) == target
    block_c = rng.integers(0, cols, _BLOCK, dtype=np.int32)
    block_v = rng.integers(-8, 8, _BLOCK).astype(np.float32)
    col_idx = np.empty(target, dtype=np.int32)
    values = np.empty(target, dtype=np.float32)
    for t, lo in enumerate(range(0, target, _BLOCK)):
        n = min(_BLOCK, target - lo)
        np.add(block_c[:n], np.int32((t * 9973) % cols), out=col_idx[lo:lo + n])
        col_idx[lo:lo + n] %= np.int32(cols)
        values[lo:lo + n] = np.roll(block_v, 977 * t)[:n]
    return HostCSR(rows, cols, row_ptr, col_idx, values, f"int32_limit_{rows}x{cols}")


def model_bytes(rows: int, cols: int, nnz: int) -> int:
    """Bytes an SpMV has to move at least: 8 per nonzero (column + value),
    4 per row_ptr entry, 4 per x entry, 4 per y entry."""
    return 8 * nnz + 4 * (rows + 1) + 4 * cols + 4 * rows
