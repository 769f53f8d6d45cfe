"""Pins for the feature oracle (O2) and the tree-walk oracle (O3).  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st
from sklearn.tree import DecisionTreeClassifier

from oracle import seer_oracle as O
from workloads import csr_gen as G

GOLD = os.path.join(os.path.dirname(__file__), "golden")
IDX = {n: i for i, n in enumerate(O.FEATURE_NAMES)}


def rp_of(lens):
    rp = np.zeros(len(lens) + 1, np.int32)
    rp[1:] = np.cumsum(np.asarray(lens, np.int64))
    return rp


def test_density_worked_example_from_paper():
    # Sec. IV-A: a row 20 elements long with five nonzeros has density 0.25
    with open(os.path.join(GOLD, "row_density_example.txt")) as fh:
        width, nz, dens = [ln for ln in fh if not ln.startswith("#")][0].split()
    F = O.features(1, int(width), rp_of([int(nz)]))
    for name in ("mean_density", "max_density", "min_density"):
        assert F["f"][IDX[name]] == np.float32(float(dens))
    assert F["f"][IDX["var_density"]] == 0.0
    assert F["f"][IDX["mean_len"]] == 5.0 and F["nnz"] == 5


def test_config1_closed_form():
    F = O.features(4096, 4096, rp_of([16] * 4096))
    assert (F["rows"], F["cols"], F["nnz"], F["max_len"], F["min_len"], F["empty_rows"]) == (4096, 4096, 65536, 16, 16, 0)
    assert F["sum_sq_len"] == 4096 * 256
    f = F["f"]
    assert f[IDX["mean_len"]] == 16 and f[IDX["var_len"]] == 0 and f[IDX["empty_frac"]] == 0
    assert f[IDX["mean_density"]] == np.float32(16 / 4096)


@pytest.mark.parametrize("n", [3, 64, 1024])
def test_config2_closed_form(n):
    A = G.laplacian_5pt(n)
    F = O.features(A.rows, A.cols, A.row_ptr)
    assert F["nnz"] == 5 * n * n - 4 * n
    assert (F["max_len"], F["min_len"], F["empty_rows"]) == (5, 3, 0)
    assert F["sum_sq_len"] == 36 + 64 * (n - 2) + 25 * (n - 2) ** 2
    assert F["f"][IDX["mean_len"]] == np.float32(5 - 4 / n)
    if n == 1024:
        assert F["sum_sq_len"] == 26_177_544 and F["f"][IDX["mean_len"]] == np.float32(4.99609375)
    # exact rational variance, rounded once
    var = Fraction(F["sum_sq_len"], n * n) - Fraction(F["nnz"], n * n) ** 2
    assert abs(float(F["f"][IDX["var_len"]]) - float(var)) <= 2.0 ** -24 * float(var)


def test_config4_empty_rows_by_construction():
    A = G.empty_poisson(80_000, 10_000, 0.3, 4.0, seed=5)
    F = O.features(A.rows, A.cols, A.row_ptr)
    assert F["empty_rows"] == 24_000 and F["min_len"] == 0
    assert F["f"][IDX["empty_frac"]] == np.float32(0.3)
    assert F["nnz"] == A.nnz


def test_variance_sign_and_transposition_mistakes_are_caught():
    # lens = [0, 4]: mean 2, population variance 4 (sample variance would be 8),
    # sum_sq 16.  rows*sum_sq - nnz^2 = 32 - 16 = 16, /rows^2 = 4.
    F = O.features(2, 8, rp_of([0, 4]))
    f = F["f"]
    assert (f[IDX["mean_len"]], f[IDX["var_len"]], f[IDX["max_len"]], f[IDX["min_len"]]) == (2, 4, 4, 0)
    assert f[IDX["empty_frac"]] == 0.5
    assert f[IDX["max_density"]] == 0.5 and f[IDX["mean_density"]] == 0.25
    assert f[IDX["var_density"]] == np.float32(4 / 64)
    assert f[IDX["rows"]] == 2 and f[IDX["cols"]] == 8 and f[IDX["nnz"]] == 4


def test_degenerate_shapes():
    F = O.features(0, 7, np.zeros(1, np.int32))
    assert F["nnz"] == 0 and F["max_len"] == 0 and F["min_len"] == 0
    assert F["f"][IDX["cols"]] == 7 and F["f"][IDX["iterations"]] == 1 and np.count_nonzero(F["f"]) == 2
    F = O.features(3, 0, np.zeros(4, np.int32))
    assert F["empty_rows"] == 3 and F["f"][IDX["empty_frac"]] == 1.0
    assert np.all(F["f"][8:12] == 0)


def test_large_values_need_wide_integers():
    # two rows near the int32 limit in total: numerator ~ 2^61 must not overflow/round early
    lens = [2**30 - 1, 2**30 - 3, 0, 1]
    F = O.features(4, 2**31 - 1, rp_of(lens))
    mean = Fraction(sum(lens), 4)
    var = Fraction(sum(l * l for l in lens), 4) - mean * mean
    assert F["sum_sq_len"] == sum(l * l for l in lens)
    assert F["f"][IDX["var_len"]] == np.float32(float(var))   # Fraction->float is correctly rounded
    assert F["f"][IDX["mean_len"]] == np.float32(float(mean))


@settings(max_examples=200, deadline=None)
@given(st.lists(st.integers(0, 5000), min_size=1, max_size=300), st.integers(1, 10**6))
def test_feature_invariants_and_numpy_crosscheck(lens, cols):
    rows = len(lens)
    F = O.features(rows, cols, rp_of(lens))
    f = F["f"].astype(np.float64)
    L = np.asarray(lens, np.float64)
    assert F["nnz"] == sum(lens) and F["max_len"] == max(lens) and F["min_len"] == min(lens)
    assert F["empty_rows"] == lens.count(0)
    assert F["sum_sq_len"] <= F["max_len"] * F["nnz"]
    rel = 2.0 ** -23
    assert f[IDX["min_len"]] <= f[IDX["mean_len"]] * (1 + rel) and f[IDX["mean_len"]] <= f[IDX["max_len"]] * (1 + rel)
    assert f[IDX["var_len"]] >= 0
    assert (f[IDX["var_len"]] == 0) == (min(lens) == max(lens))
    assert abs(f[IDX["mean_len"]] - L.mean()) <= rel * L.mean() + 1e-300
    assert abs(f[IDX["var_len"]] - L.var()) <= 1e-6 * L.var() + 1e-9 * (L.mean() ** 2)
    assert abs(f[IDX["var_density"]] - L.var() / cols**2) <= 1e-6 * L.var() / cols**2 + 1e-9 * (L.mean() / cols) ** 2
    assert abs(f[IDX["mean_density"]] - L.mean() / cols) <= rel * L.mean() / cols


# ---------------------------------------------------------------- O3: tree walk
def tree_arrays(clf):
    t = clf.tree_
    feat = np.where(t.children_left < 0, -1, t.feature).astype(np.int32)
    klass = clf.classes_[np.argmax(t.value[:, 0, :], axis=1)].astype(np.int32)
    return feat, t.threshold.astype(np.float64), t.children_left.astype(np.int32), t.children_right.astype(np.int32), klass


def test_hand_built_trees():
    # depth 0
    assert O.select(np.zeros(O.NUM_FEATURES, np.float32), [-1], [0.0], [-1], [-1], [3]) == 3
    # depth 2:  f4 <= 10 ? (f7 <= 0.5 ? 0 : 1) : 2
    feat, thr = [4, 7, -1, -1, -1], [10.0, 0.5, 0, 0, 0]
    left, right, kl = [1, 2, -1, -1, -1], [4, 3, -1, -1, -1], [-1, -1, 0, 1, 2]
    f = np.zeros(O.NUM_FEATURES, np.float32)
    f[4], f[7] = 10.0, 0.5
    assert O.select(f, feat, thr, left, right, kl) == 0      # both ties go left
    f[7] = np.nextafter(np.float32(0.5), np.float32(1))
    assert O.select(f, feat, thr, left, right, kl) == 1
    f[4] = np.nextafter(np.float32(10), np.float32(11))
    assert O.select(f, feat, thr, left, right, kl) == 2
    with pytest.raises(ValueError):
        O.select(f, [0, 0], [1e30, 1e30], [1, 0], [1, 0], [0, 0])


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_against_sklearn_predict(seed):
    rng = np.random.default_rng(seed)
    X = np.exp(rng.normal(3, 3, (600, O.NUM_FEATURES))).astype(np.float32)
    X[:, 7] = rng.random(600)
    w = rng.normal(size=O.NUM_FEATURES)
    lab = (np.log1p(X.astype(np.float64)) @ w > 0).astype(int) + 2 * (X[:, 7] > 0.5)
    clf = DecisionTreeClassifier(criterion="gini", max_depth=6, random_state=0).fit(X, lab)
    arrs = tree_arrays(clf)
    # training rows, fresh rows, and rows sitting exactly on thresholds (as fp32)
    Xt = np.exp(rng.normal(3, 3, (400, O.NUM_FEATURES))).astype(np.float32)
    on_thr = []
    feat, thr = arrs[0], arrs[1]
    for n in np.flatnonzero(feat >= 0):
        row = Xt[rng.integers(400)].copy()
        row[feat[n]] = np.float32(thr[n])
        on_thr.append(row)
        row2 = row.copy()
        row2[feat[n]] = np.nextafter(np.float32(thr[n]), np.float32(np.inf))
        on_thr.append(row2)
    allX = np.concatenate([X, Xt, np.array(on_thr, np.float32)])
    want = clf.predict(allX)
    got = np.array([O.select(r, *arrs) for r in allX])
    assert np.array_equal(got, want)


# ---------------------------------------------------------------- known features / model
def test_known_features_are_the_free_part_of_the_gathered_vector():
    # closed form (config 1) and agreement with the gathered vector wherever both are defined
    k = O.known_features(4096, 4096, 65536)
    assert (k[0], k[1], k[2], k[3]) == (4096, 4096, 65536, 16) and k[8] == np.float32(16 / 4096)
    assert np.all(k[[4, 5, 6, 7, 9, 10, 11]] == 0)
    for A in (G.laplacian_5pt(37), G.empty_poisson(5000, 300, 0.3, 4.0, seed=2), G.zipf_rows(3000, s=1.5, cap=500, seed=3)):
        f = O.features(A.rows, A.cols, A.row_ptr)["f"]
        k = O.known_features(A.rows, A.cols, A.nnz)
        assert np.array_equal(k[[0, 1, 2, 3, 8, 12]], f[[0, 1, 2, 3, 8, 12]])
    assert np.count_nonzero(O.known_features(0, 9, 0)) == 2        # cols and the iteration count


def test_model_select_hand_cases():
    # selector: rows <= 100 -> known model, else gather.  known: constant kernel 1.
    # gathered: var_len <= 5 ? 2 : 3
    selector = ([0, -1, -1], [100.0, 0, 0], [1, -1, -1], [2, -1, -1], [-1, 0, 1])
    known = ([-1], [0.0], [-1], [-1], [1])
    gathered = ([6, -1, -1], [5.0, 0, 0], [1, -1, -1], [2, -1, -1], [-1, 2, 3])
    fg = np.zeros(O.NUM_FEATURES, np.float32)
    fg[6] = 7.0
    assert O.model_select(100, 50, 10, fg, selector, known, gathered) == (0, 1)
    assert O.model_select(101, 50, 10, fg, selector, known, gathered) == (1, 3)
    fg[6] = 5.0
    assert O.model_select(101, 50, 10, fg, selector, known, gathered) == (1, 2)
    assert O.model_select(5, 50, 10, fg, None, None, gathered) == (1, 2)


def test_iteration_count_is_a_known_feature():
    """Sec. IV-E (multiple iterations): the number of iterations is available to every
    predictor.  It is the last entry of both vectors, 1 unless stated, and a tree may
    split on it."""
    rp = rp_of([1, 2, 3])
    assert O.features(3, 4, rp)["f"][IDX["iterations"]] == 1
    assert O.features(3, 4, rp, iterations=19)["f"][IDX["iterations"]] == 19
    assert np.array_equal(O.features(3, 4, rp, iterations=19)["f"][:12], O.features(3, 4, rp)["f"][:12])
    kf = O.known_features(3, 4, 6, iterations=19)
    assert kf[IDX["iterations"]] == 19 and kf[IDX["nnz"]] == 6
    # known: iterations <= 18.5 ? kernel 4 : kernel 5 (preprocessing amortised from 19 on)
    known = ([12, -1, -1], [18.5, 0, 0], [1, -1, -1], [2, -1, -1], [-1, 4, 5])
    selector = ([-1], [0.0], [-1], [-1], [0])
    fg = O.features(3, 4, rp, iterations=19)["f"]
    assert O.model_select(3, 4, 6, fg, selector, known, known, iterations=18) == (0, 4)
    assert O.model_select(3, 4, 6, fg, selector, known, known, iterations=19) == (0, 5)


# ---------------------------------------------------------------- reachable classes
def test_reachable_classes_hand_cases():
    # rows <= 100 ? (var_len <= 5 ? 2 : 3) : (nnz <= 1000 ? 1 : (max_len <= 9 ? 1 : 4))
    tree = ([0, 6, 2, -1, -1, -1, 4, -1, -1], [100.0, 5.0, 1000.0, 0, 0, 0, 9.0, 0, 0],
            [1, 3, 5, -1, -1, -1, 7, -1, -1], [2, 4, 6, -1, -1, -1, 8, -1, -1],
            [-1, -1, -1, 2, 3, 1, -1, 1, 4])
    assert O.reachable_classes(O.known_features(100, 7, 50), *tree) == {2, 3}       # on the threshold: left
    assert O.reachable_classes(O.known_features(101, 7, 1000), *tree) == {1}        # known all the way down
    assert O.reachable_classes(O.known_features(101, 7, 1001), *tree) == {1, 4}
    # both children of a gathered test end in the same class: nothing to gather for
    same = ([6, -1, -1], [5.0, 0, 0], [1, -1, -1], [2, -1, -1], [-1, 3, 3])
    assert O.reachable_classes(O.known_features(5, 5, 5), *same) == {3}
    assert O.reachable_classes(O.known_features(5, 5, 5), [-1], [0.0], [-1], [-1], [2]) == {2}


def test_reachable_classes_never_miss_what_select_returns():
    """Brute force: whatever the gathered entries are, the class select returns lies in the
    set; a tree over known entries alone leaves exactly that class; a tree over gathered
    entries alone leaves every class some vector reaches (each leaf is shown reachable by a
    vector built from its path where the path's tests on one entry do not contradict)."""
    from test_abi_host import random_tree
    rng = np.random.default_rng(31)
    gathered_idx = [i for i in range(O.NUM_FEATURES) if i not in O.KNOWN_FEATURES]
    for trial in range(60):
        arrs = random_tree(rng, int(rng.integers(1, 40)), n_classes=5)
        rows, cols = int(rng.integers(1, 10**6)), int(rng.integers(1, 10**6))
        nnz = int(rng.integers(0, 10**7))
        kf = O.known_features(rows, cols, nnz)
        reach = O.reachable_classes(kf, *arrs)
        hit = set()
        for _ in range(200):
            f = kf.copy()
            f[gathered_idx] = np.exp(rng.normal(2, 3, len(gathered_idx))).astype(np.float32)
            k = O.select(f, *arrs)
            assert k in reach, (trial, k, reach)
            hit.add(k)
        assert hit <= reach
        # only known entries tested: the set is what select answers
        feat = np.array(arrs[0])
        known_only = [int(rng.choice(O.KNOWN_FEATURES)) if v >= 0 else -1 for v in feat]
        assert O.reachable_classes(kf, known_only, *arrs[1:]) == {O.select(kf, known_only, *arrs[1:])}
        # only gathered entries tested: every leaf is possible
        gathered_only = [int(rng.choice(gathered_idx)) if v >= 0 else -1 for v in feat]
        leaves = set()
        stack = [0]
        while stack:
            n = stack.pop()
            if gathered_only[n] < 0:
                leaves.add(arrs[4][n])
            else:
                stack += [arrs[2][n], arrs[3][n]]
        assert O.reachable_classes(kf, gathered_only, *arrs[1:]) == leaves
