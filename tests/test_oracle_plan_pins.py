"""Pins of the oracle's Adaptive-CSR plan (row blocks found in a preprocessing pass,
Sec. IV).  The plan is this build's data structure, so what pins it is what any valid
plan must satisfy: executed literally it assigns every nonzero to its own row exactly
once (exact integer arithmetic against the plain row sums), blocks are bounded, and its
block boundaries agree with a brute-force restatement on tiny inputs."""
import numpy as np
import pytest

from oracle import seer_oracle as O


def random_csr(rng, rows, cols, max_len, p_empty=0.3, p_long=0.1, long_len=40):
    lens = rng.integers(0, max_len + 1, rows)
    lens[rng.random(rows) < p_empty] = 0
    lens[rng.random(rows) < p_long] = rng.integers(long_len // 2, long_len + 1)
    rp = np.zeros(rows + 1, np.int64)
    rp[1:] = np.cumsum(lens)
    nnz = int(rp[-1])
    ci = rng.integers(0, cols, nnz)
    va = rng.integers(-3, 4, nnz)
    x = rng.integers(-3, 4, cols)
    return rp, ci, va, x


def row_sums(rows, rp, ci, va, x):
    return [int(sum(int(va[j]) * int(x[ci[j]]) for j in range(rp[i], rp[i + 1]))) for i in range(rows)]


@pytest.mark.parametrize("chunk", [1, 2, 4, 8, 16])
def test_plan_executes_to_the_row_sums(chunk):
    rng = np.random.default_rng(100 + chunk)
    for trial in range(60):
        rows = int(rng.integers(1, 40))
        rp, ci, va, x = random_csr(rng, rows, 9, int(rng.integers(0, 7)))
        row, start = O.adaptive_plan(rows, rp, chunk)
        got = O.plan_spmv_python(rows, rp, ci.tolist(), [int(v) for v in va], [int(v) for v in x], row, start)
        assert got == row_sums(rows, rp, ci, va, x), (chunk, trial)


@pytest.mark.parametrize("chunk", [1, 3, 4, 8])
def test_plan_shape_invariants(chunk):
    rng = np.random.default_rng(7 + chunk)
    for trial in range(80):
        rows = int(rng.integers(1, 50))
        rp, *_ = random_csr(rng, rows, 5, int(rng.integers(0, 6)))
        nnz = int(rp[-1])
        row, start = O.adaptive_plan(rows, rp, chunk)
        n = len(row) - 1
        assert n == max(1, -(-nnz // chunk)) and len(start) == n + 1
        assert row[0] == 0 and start[0] == 0 and row[n] == rows and start[n] == nnz
        assert np.all(np.diff(row) >= 0) and np.all(np.diff(start) >= 0)
        # a block never holds more than two chunks, and never reaches back past the chunk before its own
        assert np.all(np.diff(start) <= 2 * chunk)
        for k in range(n):
            assert (k - 1) * chunk <= start[k] <= k * chunk or k == 0
            assert start[k + 1] <= (k + 1) * chunk


def test_plan_boundaries_by_brute_force():
    """row[k] restated with no search: count the rows whose end is at or before k*chunk."""
    rng = np.random.default_rng(3)
    for trial in range(50):
        rows = int(rng.integers(1, 30))
        rp, *_ = random_csr(rng, rows, 5, 5)
        chunk = int(rng.integers(1, 9))
        row, start = O.adaptive_plan(rows, rp, chunk)
        n = len(row) - 1
        for k in range(1, n):
            ending = sum(1 for i in range(rows) if rp[i + 1] <= k * chunk)
            assert row[k] == ending
            inside_one_row = k >= 1 and row[k - 1] == row[k]
            assert start[k] == (k * chunk if inside_one_row else rp[row[k]])


def test_plan_worked_cases():
    # one row of 10 nonzeros, chunk 4: three blocks, all of them inside row 0 until the last
    row, start = O.adaptive_plan(1, [0, 10], 4)
    assert row.tolist() == [0, 0, 0, 1] and start.tolist() == [0, 4, 8, 10]
    # rows of 2 nonzeros, chunk 4: blocks of exactly two rows
    row, start = O.adaptive_plan(6, [0, 2, 4, 6, 8, 10, 12], 4)
    assert row.tolist() == [0, 2, 4, 6] and start.tolist() == [0, 4, 8, 12]
    # rows of 3, chunk 4: every block begins on a row boundary before its nominal start
    row, start = O.adaptive_plan(4, [0, 3, 6, 9, 12], 4)
    assert row.tolist() == [0, 1, 2, 4] and start.tolist() == [0, 3, 6, 12]
    # leading empty rows go with block 0 even when the first nonempty row is long
    row, start = O.adaptive_plan(3, [0, 0, 0, 9], 4)
    assert row.tolist() == [0, 2, 2, 3] and start.tolist() == [0, 0, 8, 9]
    # no nonzeros at all: one block that owns every row
    row, start = O.adaptive_plan(5, [0] * 6, 4)
    assert row.tolist() == [0, 5] and start.tolist() == [0, 0]
    # rows == 0
    row, start = O.adaptive_plan(0, [0], 4)
    assert row.tolist() == [0] and start.tolist() == [0]


def test_planted_mistakes_are_caught():
    """The executor catches a plan that is off by one in either array.  (A split point
    inside one long row may move freely, so only starts on a row boundary are moved.)"""
    rp = np.array([0, 3, 3, 11, 12, 20], np.int64)
    rng = np.random.default_rng(1)
    ci = rng.integers(0, 4, 20).tolist()
    va = [1] * 20
    x = [1, 2, 3, 5]
    want = row_sums(5, rp, ci, va, x)
    row, start = O.adaptive_plan(5, rp, 4)
    assert O.plan_spmv_python(5, rp, ci, va, x, row, start) == want
    for arr in ("row", "start"):
        for k in range(1, len(row) - 1):
            if arr == "start" and start[k] != rp[row[k]]:
                continue
            r2, s2 = row.copy(), start.copy()
            (r2 if arr == "row" else s2)[k] += 1
            try:
                got = O.plan_spmv_python(5, rp, ci, va, x, r2, s2)
            except IndexError:
                continue                      # ran off the matrix: caught as well
            assert got != want, (arr, k)
