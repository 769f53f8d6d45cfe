"""Pins for the oracle's count of CSR contract violations: cases whose counts follow
from how they are built."""
import numpy as np

from oracle import seer_oracle as O
from workloads import csr_gen as G


def i32(*v):
    return np.array(v, dtype=np.int32)


def test_well_formed_matrices_have_no_defects():
    for A in (G.laplacian_5pt(12), G.fixed_degree(64, 64, 4, seed=3), G.explicit_lengths([0, 0, 7, 0, 1], 9, seed=1)):
        assert O.csr_defects(A.rows, A.cols, A.nnz, A.row_ptr, A.col_idx) == (0, 0)
    assert O.csr_defects(0, 5, 0, i32(0), i32()) == (0, 0)           # no rows
    assert O.csr_defects(3, 0, 0, i32(0, 0, 0, 0), i32()) == (0, 0)   # no columns, no entries


def test_each_kind_of_offset_defect_counts_once():
    ci = i32(0, 1, 2, 3)
    assert O.csr_defects(2, 4, 4, i32(0, 2, 4), ci) == (0, 0)
    assert O.csr_defects(2, 4, 4, i32(1, 2, 4), ci) == (1, 0)        # does not start at 0
    assert O.csr_defects(2, 4, 4, i32(0, 2, 3), ci) == (1, 0)        # does not end at nnz
    assert O.csr_defects(2, 4, 4, i32(0, 5, 4), ci) == (1, 0)        # one descent (5 -> 4)
    assert O.csr_defects(3, 4, 4, i32(0, 3, 1, 4), ci) == (1, 0)     # a descent in the middle, ends right
    assert O.csr_defects(3, 4, 4, i32(2, 1, 0, 3), ci) == (4, 0)     # start, two descents, end
    assert O.csr_defects(2, 4, 4, i32(0, -1, 4), ci) == (1, 0)       # a negative offset is a descent


def test_column_defects_count_entries_outside_the_columns():
    rp = i32(0, 3, 6)
    assert O.csr_defects(2, 4, 6, rp, i32(0, 3, 2, 1, 0, 3)) == (0, 0)
    assert O.csr_defects(2, 4, 6, rp, i32(0, 4, 2, 1, 0, 3)) == (0, 1)   # == cols
    assert O.csr_defects(2, 4, 6, rp, i32(-1, 4, 2, 1, 0, 7)) == (0, 3)  # negative, == cols, beyond
    assert O.csr_defects(2, 0, 6, rp, i32(0, 0, 0, 0, 0, 0)) == (0, 6)   # no columns: every entry is outside
    # only the first nnz entries are the matrix's
    assert O.csr_defects(2, 4, 3, i32(0, 3, 3), i32(0, 1, 2, 99, -5)) == (0, 0)


def test_planted_defects_in_a_larger_matrix_are_counted_exactly():
    A = G.random_lengths(5000, 700, 0, 9, seed=11)
    rng = np.random.default_rng(5)
    ci = A.col_idx.copy()
    where = rng.choice(A.nnz, 37, replace=False)
    ci[where[:20]] = A.cols + rng.integers(0, 1000, 20)
    ci[where[20:]] = -1 - rng.integers(0, 1000, 17)
    rp = A.row_ptr.copy()
    lens = np.diff(rp)
    # raise an offset above its successor: row i longer than it is, the next pair descends
    # (rows spaced out so that the planted descents do not touch each other)
    rows_hit = [i for i in range(10, 4000, 400) if lens[i] > 0][:8]
    for i in rows_hit:
        rp[i] = rp[i + 1] + 1
    bad_rp, bad_ci = O.csr_defects(A.rows, A.cols, A.nnz, rp, ci)
    assert bad_ci == 37
    assert bad_rp == len(rows_hit)
