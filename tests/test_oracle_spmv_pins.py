"""Pins for the SpMV oracle (O1): it is checked against things that are not itself --
dense brute force, identities, closed forms of the 5-point Laplacian, a library
routine, invariants -- so that a dropped term, wrong index or transposed operand
fails at least one test.  CPU only."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import seer_oracle as O
from workloads import csr_gen as G


def dense_of(A: G.HostCSR) -> np.ndarray:
    """Dense fp64 copy, duplicates summed, built entry by entry."""
    D = np.zeros((A.rows, A.cols), dtype=np.float64)
    for i in range(A.rows):
        for k in range(A.row_ptr[i], A.row_ptr[i + 1]):
            D[i, A.col_idx[k]] += float(A.values[k])
    return D


def tiny_cases():
    cases = []
    cases.append(G.explicit_lengths([], 5, 1, "0x5"))
    cases.append(G.explicit_lengths([0, 0, 0], 4, 2, "all-empty"))
    cases.append(G.explicit_lengths([1], 1, 3, "1x1"))
    cases.append(G.explicit_lengths([0, 7, 0, 0, 3, 0], 7, 4, "empties+full-row"))
    cases.append(G.explicit_lengths([64] + [0] * 10, 64, 5, "one-full-row"))
    cases.append(G.explicit_lengths([9] * 6, 3, 6, "duplicates (len > cols)"))
    for s in range(8):
        rows, cols = 1 + 7 * s, 1 + 5 * ((s * 3) % 9)
        cases.append(G.random_lengths(rows, cols, 0, min(cols, 9), 100 + s))
    cases.append(G.random_lengths(40, 64, 0, 64, 200))
    return cases


@pytest.mark.parametrize("A", tiny_cases(), ids=lambda a: a.name)
def test_matches_dense_brute_force(A):
    A.validate()
    x = G.dense_vector(A.cols, 11)
    y, b = O.spmv(A.rows, A.row_ptr, A.col_idx, A.values, x)
    D = dense_of(A)
    y_dense = np.array([sum(D[i, j] * float(x[j]) for j in range(A.cols)) for i in range(A.rows)])
    # dense sums the same exact products in another order: agree to a few ulp of the bound
    Dabs = np.zeros_like(D)
    for i in range(A.rows):
        for k in range(A.row_ptr[i], A.row_ptr[i + 1]):
            Dabs[i, A.col_idx[k]] += abs(float(A.values[k]))
    b_dense = Dabs @ np.abs(x.astype(np.float64))
    assert y.shape == (A.rows,)
    assert np.all(np.abs(y - y_dense) <= 1e-12 * (b_dense + 1e-300))
    assert np.allclose(b, b_dense, rtol=1e-12, atol=0)
    # pure-Python row loop: same order of operations, must be identical
    y2, b2 = O.spmv_python(A.rows, A.row_ptr, A.col_idx, A.values, x)
    assert np.array_equal(y, y2) and np.array_equal(b, b2)


def test_non_symmetric_catches_transposed_gather():
    # A = e_0 e_2^T : y_0 = x_2.  Using x[row] or A^T would give something else.
    rp = np.array([0, 1, 1, 1], np.int32)
    ci = np.array([2], np.int32)
    va = np.array([1.0], np.float32)
    x = np.array([10.0, 20.0, 30.0], np.float32)
    y, b = O.spmv(3, rp, ci, va, x)
    assert y.tolist() == [30.0, 0.0, 0.0] and b.tolist() == [30.0, 0.0, 0.0]


def test_identity_and_diagonal_exact():
    n = 1000
    rp = np.arange(n + 1, dtype=np.int32)
    ci = np.arange(n, dtype=np.int32)
    x = G.dense_vector(n, 3)
    y, _ = O.spmv(n, rp, ci, np.ones(n, np.float32), x)
    assert np.array_equal(y, x.astype(np.float64))
    d = G.dense_vector(n, 4)
    y, b = O.spmv(n, rp, ci, d, x)
    assert np.array_equal(y, d.astype(np.float64) * x.astype(np.float64))  # exact in fp64
    assert np.array_equal(b, np.abs(y))
    # permuted diagonal: y_i = d_i * x[p_i]
    p = np.random.default_rng(5).permutation(n).astype(np.int32)
    y, _ = O.spmv(n, rp, p, d, x)
    assert np.array_equal(y, d.astype(np.float64) * x[p].astype(np.float64))


def test_row_sums_for_x_equal_one():
    A = G.small_integer_values(G.random_lengths(500, 300, 0, 40, 21), 22)
    x = np.ones(A.cols, np.float32)
    y, b = O.spmv(A.rows, A.row_ptr, A.col_idx, A.values, x)
    sums = np.add.reduceat(np.concatenate([A.values.astype(np.float64), [0.0]]),
                           np.minimum(A.row_ptr[:-1], A.nnz))
    sums[np.diff(A.row_ptr) == 0] = 0.0
    assert np.array_equal(y, sums)
    assert np.all(b >= np.abs(y))


@pytest.mark.parametrize("maker", [
    lambda: G.fixed_degree(256, 256, 16, seed=9),
    lambda: G.random_lengths(3000, 1000, 0, 30, 31),
    lambda: G.zipf_rows(5000, s=1.6, cap=2000, seed=32),
    lambda: G.empty_poisson(20000, 5000, 0.3, 4.0, seed=33),
    lambda: G.banded(777, 5, 34),
])
def test_against_scipy_fp64(maker):
    A = maker()
    A.validate()
    x = G.dense_vector(A.cols, 77)
    y, b = O.spmv(A.rows, A.row_ptr, A.col_idx, A.values, x)
    M = sp.csr_matrix((A.values.astype(np.float64), A.col_idx, A.row_ptr), shape=(A.rows, A.cols))
    ys = M.dot(x.astype(np.float64))
    Mabs = sp.csr_matrix((np.abs(A.values).astype(np.float64), A.col_idx, A.row_ptr), shape=(A.rows, A.cols))
    bs = Mabs.dot(np.abs(x).astype(np.float64))
    assert np.all(np.abs(y - ys) <= 1e-13 * bs + 1e-300)
    assert np.allclose(b, bs, rtol=1e-13, atol=0)


@pytest.mark.parametrize("n", [2, 3, 17, 64])
def test_laplacian_closed_forms(n):
    A = G.laplacian_5pt(n)
    A.validate()
    assert A.nnz == 5 * n * n - 4 * n
    # x = 1: y = 4 - (number of neighbours) = 0 interior, 1 edge, 2 corner
    y, b = O.spmv(A.rows, A.row_ptr, A.col_idx, A.values, np.ones(A.cols, np.float32))
    r, c = np.divmod(np.arange(n * n), n)
    on_edge = ((r == 0) | (r == n - 1)).astype(int) + ((c == 0) | (c == n - 1)).astype(int)
    assert np.array_equal(y, on_edge.astype(np.float64))
    assert np.array_equal(b, 8.0 - on_edge)
    # Dirichlet eigenvectors: x_{r,c} = sin(pi p (r+1)/(n+1)) sin(pi q (c+1)/(n+1)),
    # A x = (4 - 2cos(pi p/(n+1)) - 2cos(pi q/(n+1))) x
    for p, q in [(1, 1), (2, 1), (n, n)]:
        xe = (np.sin(np.pi * p * (r + 1) / (n + 1)) * np.sin(np.pi * q * (c + 1) / (n + 1))).astype(np.float32)
        lam = 4 - 2 * np.cos(np.pi * p / (n + 1)) - 2 * np.cos(np.pi * q / (n + 1))
        y, b = O.spmv(A.rows, A.row_ptr, A.col_idx, A.values, xe)
        # xe was rounded to fp32 (relative 6e-8 per entry), the oracle itself is fp64
        assert np.all(np.abs(y - lam * xe.astype(np.float64)) <= 2.0 ** -23 * b + 1e-300)


def test_full_size_laplacian_counts():
    A = G.laplacian_5pt(1024)
    assert A.rows == 1_048_576 and A.nnz == 5_238_784
    y, _ = O.spmv(A.rows, A.row_ptr, A.col_idx, A.values, np.ones(A.cols, np.float32))
    vals, cnt = np.unique(y, return_counts=True)
    assert vals.tolist() == [0.0, 1.0, 2.0]
    assert cnt.tolist() == [1022 * 1022, 4 * 1022, 4]


def test_row_permutation_and_in_row_shuffle():
    A = G.random_lengths(400, 300, 0, 25, 41)
    x = G.dense_vector(A.cols, 42)
    y, b = O.spmv(A.rows, A.row_ptr, A.col_idx, A.values, x)
    rng = np.random.default_rng(43)
    perm = rng.permutation(A.rows)
    lens = np.diff(A.row_ptr)
    rp2 = np.zeros(A.rows + 1, np.int32)
    rp2[1:] = np.cumsum(lens[perm])
    ci2 = np.concatenate([A.col_idx[A.row_ptr[i]:A.row_ptr[i + 1]] for i in perm] + [np.zeros(0, np.int32)])
    va2 = np.concatenate([A.values[A.row_ptr[i]:A.row_ptr[i + 1]] for i in perm] + [np.zeros(0, np.float32)])
    y2, b2 = O.spmv(A.rows, rp2, ci2, va2, x)
    assert np.array_equal(y2, y[perm]) and np.array_equal(b2, b[perm])
    # shuffle entries inside each row: same terms, other order
    ci3, va3 = A.col_idx.copy(), A.values.copy()
    for i in range(A.rows):
        s, e = A.row_ptr[i], A.row_ptr[i + 1]
        p = rng.permutation(e - s)
        ci3[s:e], va3[s:e] = ci3[s:e][p], va3[s:e][p]
    y3, b3 = O.spmv(A.rows, A.row_ptr, ci3, va3, x)
    assert np.all(np.abs(y3 - y) <= 1e-13 * b + 1e-300)


def test_linearity():
    A = G.random_lengths(300, 200, 0, 20, 51)
    x1 = G.dense_vector(A.cols, 52)
    x2 = G.dense_vector(A.cols, 53)
    xs = (x1.astype(np.float64) + 2.0 * x2.astype(np.float64))
    # keep xs exactly representable: use small integers instead
    x1 = np.round(x1 * 8).astype(np.float32)
    x2 = np.round(x2 * 8).astype(np.float32)
    Ai = G.small_integer_values(A, 54)
    y1, _ = O.spmv(Ai.rows, Ai.row_ptr, Ai.col_idx, Ai.values, x1)
    y2, _ = O.spmv(Ai.rows, Ai.row_ptr, Ai.col_idx, Ai.values, x2)
    y12, _ = O.spmv(Ai.rows, Ai.row_ptr, Ai.col_idx, Ai.values, (x1 + 2 * x2).astype(np.float32))
    assert np.array_equal(y12, y1 + 2 * y2)  # all integers: exact
    del xs


def test_nonnegative_inputs_bound_equals_value():
    A = G.random_lengths(200, 200, 0, 30, 61)
    A.values[:] = np.abs(A.values)
    x = np.abs(G.dense_vector(A.cols, 62))
    y, b = O.spmv(A.rows, A.row_ptr, A.col_idx, A.values, x)
    assert np.array_equal(y, b)


def test_all_cores_copy_of_the_row_loop_equals_the_single_thread_loop():
    """The OpenMP copy of the row loop (timed as a CPU baseline, never checked against) sums
    every row in the same order as the single-thread loop: bit-identical results."""
    A = G.zipf_rows(30_011, s=1.5, cap=4000, seed=41)
    x = G.dense_vector(A.cols, 42)
    y, _ = O.spmv(A.rows, A.row_ptr, A.col_idx, A.values, x, want_bound=False)
    y_all, threads = O.spmv_all_cores(A.rows, A.row_ptr, A.col_idx, A.values, x)
    assert threads >= 1 and y_all.tobytes() == y.tobytes()
