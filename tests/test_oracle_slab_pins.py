"""Pins of the oracle's column-slab plan (oracle.slab_plan): a worked case, brute-force
restatements on small random matrices, the literal product from the plan, and the cases in
which the form does not apply."""
import numpy as np
import pytest

from oracle import seer_oracle as O
from workloads import csr_gen as G


def small(seed, rows=40, cols=70, lo=0, hi=9):
    A = G.random_lengths(rows, cols, lo, hi, seed)
    return A


def test_worked_case():
    # 3 rows, 8 columns, slabs of 4 columns (shift 2):
    # row 0: cols 1 5 6 | row 1: (empty) | row 2: cols 0 3 4
    rp = np.array([0, 3, 3, 6], np.int32)
    ci = np.array([1, 5, 6, 0, 3, 4], np.int32)
    p = O.slab_plan(3, 8, rp, ci, shift=2)
    assert p["n_slabs"] == 2
    # slab 0: row 0 {1}, row 1 {}, row 2 {0, 3}; slab 1: row 0 {5, 6}, row 1 {}, row 2 {4}
    assert p["rp_v"].tolist() == [0, 1, 1, 3, 5, 5, 6]
    assert p["perm"].tolist() == [0, 3, 4, 1, 2, 5]
    # kept: virtual rows 0, 2, 3, 5; row 0 owns kept rows 0 and 2, row 1 none, row 2 owns 1 and 3
    assert p["rp_z"].tolist() == [0, 1, 3, 5, 6]
    assert p["rp_j"].tolist() == [0, 2, 2, 4] and p["p_idx"].tolist() == [0, 2, 1, 3]


def test_brute_force_restatement():
    """Each virtual row, listed by looping over the matrix the slow way, is what the plan says."""
    for seed in range(12):
        A = small(seed, rows=23 + seed, cols=50 + 3 * seed)
        shift = 2 + seed % 3
        p = O.slab_plan(A.rows, A.cols, A.row_ptr, A.col_idx, shift)
        S = -(-A.cols // (1 << shift))
        assert p is not None and p["n_slabs"] == S
        want_perm, want_rp = [], [0]
        for s in range(S):
            for i in range(A.rows):
                for k in range(int(A.row_ptr[i]), int(A.row_ptr[i + 1])):
                    if int(A.col_idx[k]) // (1 << shift) == s:
                        want_perm.append(k)
                want_rp.append(len(want_perm))
        assert p["perm"].tolist() == want_perm and p["rp_v"].tolist() == want_rp
        assert sorted(want_perm) == list(range(A.nnz))            # every entry exactly once
        # the kept rows and each row's pieces, the slow way
        kept = [v for v in range(S * A.rows) if want_rp[v + 1] > want_rp[v]]
        assert p["rp_z"].tolist() == [want_rp[v] for v in kept] + [A.nnz]
        pieces = [[j for j, v in enumerate(kept) if v % A.rows == i] for i in range(A.rows)]
        assert p["p_idx"].tolist() == [j for pc in pieces for j in pc]
        assert p["rp_j"].tolist() == [0] + list(np.cumsum([len(pc) for pc in pieces]))


def test_literal_product_equals_row_sums():
    rng = np.random.default_rng(5)
    for seed in range(6):
        A = small(100 + seed, rows=31, cols=90, hi=14)
        vals = rng.integers(-4, 5, A.nnz).astype(np.int64)
        x = rng.integers(-3, 4, A.cols).astype(np.int64)
        p = O.slab_plan(A.rows, A.cols, A.row_ptr, A.col_idx, shift=3 + seed % 3)
        got = O.slab_spmv_python(A.rows, p, A.col_idx, vals.tolist(), x.tolist())
        want = [int(sum(vals[k] * x[A.col_idx[k]] for k in range(A.row_ptr[i], A.row_ptr[i + 1]))) for i in range(A.rows)]
        assert got == want
        # and a planted mistake is caught: one offset moved by one hands an entry to the wrong piece
        bad = dict(p)
        bad["rp_z"] = p["rp_z"].copy()
        j = next(j for j in range(1, len(p["rp_z"]) - 1) if p["rp_z"][j] - p["rp_z"][j - 1] > 0)
        bad["rp_z"][j] -= 1                               # the last entry of kept row j - 1 now counts for kept row j
        k = int(p["perm"][bad["rp_z"][j]])
        owners = {int(pj): i for i in range(A.rows) for pj in p["p_idx"][p["rp_j"][i]:p["rp_j"][i + 1]]}
        if vals[k] * x[A.col_idx[k]] != 0 and owners[j] != owners[j - 1]:
            assert O.slab_spmv_python(A.rows, bad, A.col_idx, vals.tolist(), x.tolist()) != want


def test_where_the_form_does_not_apply():
    A = small(7)
    assert O.slab_plan(A.rows, A.cols, A.row_ptr, A.col_idx, shift=7) is None      # 70 columns: one slab
    assert O.slab_plan(0, 100, np.zeros(1, np.int32), np.zeros(0, np.int32), shift=2) is None
    # a row whose columns descend somewhere
    rp = np.array([0, 3, 5], np.int32)
    assert O.slab_plan(2, 16, rp, np.array([1, 9, 4, 2, 3], np.int32), shift=2) is None
    assert O.slab_plan(2, 16, rp, np.array([1, 4, 9, 2, 3], np.int32), shift=2) is not None   # a descent across rows is fine
    assert O.slab_plan(2, 16, rp, np.array([1, 4, 4, 3, 3], np.int32), shift=2) is not None   # repeats ascend
    # too many virtual rows for 32-bit offsets (decided from the sizes alone)
    assert O.slab_plan(2 ** 20, 2 ** 20 * 8, np.zeros(2 ** 20 + 1, np.int32), np.zeros(0, np.int32), shift=12) is None


def test_default_slab_is_two_mebibytes_of_x():
    assert (1 << O.SLAB_SHIFT) * 4 == 2 << 20
    A = G.HostCSR(3, (1 << 20) + 1, np.array([0, 1, 2, 3], np.int32), np.array([5, 1 << 19, 1 << 20], np.int32),
                  np.ones(3, np.float32), "three-slabs")
    p = O.slab_plan(A.rows, A.cols, A.row_ptr, A.col_idx)
    assert p["n_slabs"] == 3 and p["rp_v"].tolist() == [0, 1, 1, 1, 1, 2, 2, 2, 2, 3] and p["perm"].tolist() == [0, 1, 2]
    assert p["rp_z"].tolist() == [0, 1, 2, 3] and p["rp_j"].tolist() == [0, 1, 2, 3] and p["p_idx"].tolist() == [0, 1, 2]


def test_slab_width_rule():
    """2^19 columns per slab, 2^20 where at least four slabs would hold fewer than three entries
    per piece of a row: hand cases on both sides of each condition, and the BASELINE shapes."""
    four = 4 << 19
    assert O.slab_shift_for(10, four, 119) == 20          # 119 < 3 * 4 * 10
    assert O.slab_shift_for(10, four, 120) == 19
    assert O.slab_shift_for(10, four - (1 << 19), 1) == 19   # three slabs: never
    assert O.slab_shift_for(10, four + 1, 149) == 20      # five slabs: 149 < 150
    assert O.slab_shift_for(0, four, 0) == 19
    assert O.slab_shift_for(2_000_000, 2_000_000, 46_532_889) == 19      # config 3: four slabs, 23 per row
    assert O.slab_shift_for(8_000_000, 1_000_000, 22_818_339) == 19      # config 4: two slabs
    assert O.slab_shift_for(7_994_277, 7_994_277, 187_889_578) == 20     # 16 slabs, 23.5 per row
