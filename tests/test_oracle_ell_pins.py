"""Pins of the oracle's ELL conversion (the preprocessing of ELL,TM, Table II): the format
is lossless (CSR comes back entry for entry), multiplying from it gives the plain row sums
exactly on integer data, padding is inert, and the shape is what the header states."""
import numpy as np

from oracle import seer_oracle as O
from workloads import csr_gen as G


def csr_back(rows, cols, vals):
    rp, ci, va = [0], [], []
    for i in range(rows):
        for j in range(cols.shape[0]):
            if cols[j, i] >= 0:
                ci.append(int(cols[j, i]))
                va.append(float(vals[j, i]))
        rp.append(len(ci))
    return np.array(rp), np.array(ci, dtype=np.int64), np.array(va, dtype=np.float32)


def test_round_trip_and_shape():
    for A in (G.random_lengths(203, 50, 0, 9, 1), G.explicit_lengths([0, 3, 0, 1, 7], 9, 2, "t"),
              G.laplacian_5pt(7), G.explicit_lengths([0, 0, 0], 4, 3, "empty")):
        cols, vals = O.ell_from_csr(A.rows, A.row_ptr, A.col_idx, A.values)
        width = int(np.diff(A.row_ptr).max())
        assert cols.shape == vals.shape == (width, -(-A.rows // 64) * 64)
        assert cols.dtype == np.int32 and vals.dtype == np.float32
        assert int((cols >= 0).sum()) == A.nnz and np.all(vals[cols < 0] == 0)
        assert np.all(cols[:, A.rows:] == -1)
        # entries of a row sit in its first len slots, in CSR order
        lens = np.diff(A.row_ptr)
        assert np.array_equal((cols[:, :A.rows] >= 0).sum(axis=0), lens)
        for i in range(A.rows):
            assert np.all(cols[: lens[i], i] >= 0)
        rp, ci, va = csr_back(A.rows, cols, vals)
        assert np.array_equal(rp, A.row_ptr) and np.array_equal(ci, A.col_idx) and np.array_equal(va, A.values)


def test_product_from_ell_is_the_row_sum():
    A = G.small_integer_values(G.random_lengths(120, 40, 0, 12, 5), 6)
    x = np.round(G.dense_vector(A.cols, 7) * 4).astype(np.float32)
    cols, vals = O.ell_from_csr(A.rows, A.row_ptr, A.col_idx, A.values)
    y = O.ell_spmv_python(A.rows, cols, vals, [float(v) for v in x])
    y_ref, _ = O.spmv(A.rows, A.row_ptr, A.col_idx, A.values, x)
    assert np.array_equal(np.array(y, dtype=np.float64), y_ref)     # integers: exact


def test_worked_case_and_inert_padding():
    # [[a, 0, b], [0, 0, 0], [0, c, 0]]: width 2, columns stored down the rows
    cols, vals = O.ell_from_csr(3, [0, 2, 2, 3], np.array([0, 2, 1]), np.array([1.5, -2.0, 4.0], np.float32))
    assert cols[:, :3].tolist() == [[0, -1, 1], [2, -1, -1]]
    assert vals[:, :3].tolist() == [[1.5, 0.0, 4.0], [-2.0, 0.0, 0.0]]
    y = O.ell_spmv_python(3, cols, vals, [float("inf"), 2.0, 1.0])
    assert y == [float("inf"), 0, 8.0]           # the padded slots never touch x


# ---------------------------------------------------------------- COO
def test_coo_rows_invariants_and_round_trip():
    for A in (G.random_lengths(203, 50, 0, 9, 1), G.explicit_lengths([0, 3, 0, 1, 7, 0], 9, 2, "t"),
              G.laplacian_5pt(7), G.explicit_lengths([0, 0, 0], 4, 3, "empty")):
        r = O.coo_rows_from_csr(A.rows, A.row_ptr)
        assert r.dtype == np.int32 and r.shape == (A.nnz,)
        assert np.all(np.diff(r) >= 0)                                     # CSR order
        assert np.array_equal(np.bincount(r, minlength=A.rows), np.diff(A.row_ptr))   # row_ptr comes back
        # restated without slices: nonzero k belongs to the row whose range holds k
        for k in range(0, A.nnz, max(1, A.nnz // 50)):
            assert A.row_ptr[r[k]] <= k < A.row_ptr[r[k] + 1]


def test_product_from_coo_is_the_row_sum():
    A = G.small_integer_values(G.random_lengths(150, 40, 0, 12, 8), 9)
    x = np.round(G.dense_vector(A.cols, 10) * 4).astype(np.float32)
    r = O.coo_rows_from_csr(A.rows, A.row_ptr)
    y = O.coo_spmv_python(A.rows, r, A.col_idx, [float(v) for v in A.values], [float(v) for v in x])
    y_ref, _ = O.spmv(A.rows, A.row_ptr, A.col_idx, A.values, x)
    assert np.array_equal(np.array(y, dtype=np.float64), y_ref)
    assert O.coo_rows_from_csr(3, [0, 2, 2, 3]).tolist() == [0, 0, 2]
