"""CPU-only tests of the C ABI: every declared symbol is exported, host-only calls
(feature derivation, tree walk) agree bit for bit with the oracle, and argument
errors are reported as status codes.  No GPU work is issued here."""
import ctypes as C
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import paper_2403_17017_amd as S
from paper_2403_17017_amd import binding as B
from oracle import seer_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "seer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(seer_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = declared_functions()
    assert {"seer_features", "seer_select", "seer_spmv"} <= set(names)
    L = S.lib()
    for n in names:
        assert hasattr(L, n), f"{n} declared in include/seer.h but not exported"


def test_struct_layouts_match_header():
    assert C.sizeof(B.seer_csr) == 40
    assert C.sizeof(B.seer_features_t) == 7 * 8 + 13 * 4 + 4      # 13 floats, padded to 8
    assert C.sizeof(B.seer_plan) == 6 * 4 + 8 + 8 and B.seer_plan.device.offset == 24
    assert C.sizeof(B.seer_node) == 24 and B.seer_node.threshold.offset == 16
    assert C.sizeof(B.seer_tree) == 24


def test_names_and_errors():
    assert S.lib().seer_num_kernels() == 9 == S.NUM_KERNELS
    assert [S.kernel_name(k) for k in range(9)] == ["CSR,TM", "CSR,WM", "CSR,BM", "CSR,MP", "CSR,WO", "CSR,A", "ELL,TM", "COO,WM", "CSR,S"]
    assert S.lib().seer_kernel_name(9) is None
    assert S.strerror(0) == "ok" and "tree" in S.strerror(-3)
    with pytest.raises(S.SeerError):
        S.set_tuning("no_such_knob", 1)


def test_feature_names_agree():
    assert tuple(S.FEATURE_NAMES) == tuple(O.FEATURE_NAMES) and S.NUM_FEATURES == O.NUM_FEATURES


@settings(max_examples=300, deadline=None)
@given(st.lists(st.integers(0, 2**20), min_size=1, max_size=200), st.integers(0, 2**31 - 1))
def test_derivation_bit_exact_vs_oracle(lens, cols):
    rows = len(lens)
    rp = np.zeros(rows + 1, np.int64)
    rp[1:] = np.cumsum(lens)
    if rp[-1] >= 2**31:
        return
    want = O.features(rows, cols, rp.astype(np.int32))
    got = S.seer_derive_features(rows, cols, want["nnz"], want["max_len"], want["min_len"],
                                 want["empty_rows"], want["sum_sq_len"])
    assert got.vector().tobytes() == want["f"].tobytes()


def test_derivation_extremes():
    # widest numerator: two rows of ~2^30
    lens = [2**30 - 1, 2**30 - 3, 0, 1]
    rp = np.zeros(5, np.int64)
    rp[1:] = np.cumsum(lens)
    want = O.features(4, 2**31 - 1, rp.astype(np.int32))
    got = S.seer_derive_features(4, 2**31 - 1, want["nnz"], want["max_len"], want["min_len"],
                                 want["empty_rows"], want["sum_sq_len"])
    assert got.vector().tobytes() == want["f"].tobytes()
    # rows == 0 and cols == 0
    z = S.seer_derive_features(0, 9, 0, 0, 0, 0, 0)
    assert z.vector().tobytes() == O.features(0, 9, np.zeros(1, np.int32))["f"].tobytes()
    z = S.seer_derive_features(3, 0, 0, 0, 0, 3, 0)
    assert z.vector().tobytes() == O.features(3, 0, np.zeros(4, np.int32))["f"].tobytes()
    with pytest.raises(S.SeerError):
        S.seer_derive_features(2, 2, 10, 1, 0, 0, 1)   # rows*sum_sq < nnz^2: impossible
    with pytest.raises(S.SeerError):
        S.seer_derive_features(-1, 2, 0, 0, 0, 0, 0)


def test_known_features():
    f = S.seer_known_features(1000, 2000, 30000)
    v = f.vector()
    assert v[0] == 1000 and v[1] == 2000 and v[2] == 30000
    assert v[3] == 30 and v[8] == np.float32(30 / 2000)
    assert np.all(v[[4, 5, 6, 7, 9, 10, 11]] == 0)


@settings(max_examples=300, deadline=None)
@given(st.integers(0, 2**31 - 1), st.integers(0, 2**31 - 1), st.integers(0, 2**31 - 1))
def test_known_features_bit_exact_vs_oracle(rows, cols, nnz):
    got = S.seer_known_features(rows, cols, nnz).vector()
    assert got.tobytes() == O.known_features(rows, cols, nnz).tobytes()


def random_tree(rng, n_internal, n_classes=4):
    """Random binary tree in preorder, as parallel arrays."""
    feat, thr, left, right, kl = [], [], [], [], []

    def grow(budget):
        me = len(feat)
        feat.append(-1); thr.append(0.0); left.append(-1); right.append(-1); kl.append(int(rng.integers(n_classes)))
        if budget > 0:
            feat[me] = int(rng.integers(O.NUM_FEATURES))
            thr[me] = float(np.float32(np.exp(rng.normal(2, 3)))) if rng.random() < 0.5 else float(np.exp(rng.normal(2, 3)))
            kl[me] = -1
            lb = int(rng.integers(0, budget))
            left[me] = grow(lb)
            right[me] = grow(budget - 1 - lb)
        return me

    grow(n_internal)
    return feat, thr, left, right, kl


def test_tree_reachable_matches_oracle():
    """seer_tree_reachable against the oracle's definition: random trees (also ones whose nodes
    share children), random sizes, sizes that sit exactly on a threshold, an iteration count."""
    rng = np.random.default_rng(404)
    for trial in range(300):
        feat, thr, left, right, kl = random_tree(rng, int(rng.integers(0, 60)), n_classes=8)
        rows, cols, nnz = int(rng.integers(1, 10**7)), int(rng.integers(1, 10**7)), int(rng.integers(0, 10**8))
        kf = S.seer_known_features(rows, cols, nnz)
        if trial % 3 == 0:
            kf.f[12] = float(rng.integers(1, 100))
        want_f = np.array(list(kf.f), np.float32)
        internal = [i for i, f in enumerate(feat) if f >= 0]
        if internal and trial % 2 == 0:                    # put a known value exactly on a threshold
            n = internal[int(rng.integers(len(internal)))]
            feat[n] = int(rng.choice(O.KNOWN_FEATURES))
            thr[n] = float(want_f[feat[n]])
        if len(internal) > 2 and trial % 5 == 0:           # two parents, one child
            left[internal[-1]] = left[internal[0]] if internal[0] != internal[-1] else left[internal[-1]]
        tree = S.Tree(feat, thr, left, right, kl, n_classes=8)
        assert S.seer_tree_reachable(tree, kf) == O.reachable_classes(want_f, feat, thr, left, right, kl), trial
    # a tree over known features only: exactly what seer_select answers
    t = S.Tree([0, 2, -1, -1, -1], [1000.0, 5e4, 0, 0, 0], [1, 2, -1, -1, -1], [4, 3, -1, -1, -1], [-1, -1, 0, 1, 2])
    kf = S.seer_known_features(1000, 10, 50001)
    assert S.seer_tree_reachable(t, kf) == {S.seer_select(kf, t)} == {1}
    with pytest.raises(S.SeerError):                        # malformed: child out of range
        S.seer_tree_reachable(S.Tree([0, -1], [1.0, 0], [1, -1], [7, -1], [-1, 0]), kf)



@pytest.mark.parametrize("seed", range(6))
def test_select_bit_exact_vs_oracle(seed):
    rng = np.random.default_rng(seed)
    arrs = random_tree(rng, n_internal=int(rng.integers(0, 40)))
    tree = S.Tree(*arrs)
    thr = [t for f, t in zip(arrs[0], arrs[1]) if f >= 0]
    for _ in range(300):
        f = B.seer_features_t()
        vec = np.exp(rng.normal(2, 3, O.NUM_FEATURES)).astype(np.float32)
        if thr and rng.random() < 0.5:      # sit exactly on a threshold
            vec[int(rng.integers(O.NUM_FEATURES))] = np.float32(thr[int(rng.integers(len(thr)))])
        for i in range(O.NUM_FEATURES):
            f.f[i] = float(vec[i])
        assert S.seer_select(f, tree) == O.select(vec, *arrs)


def test_select_against_sklearn_tree():
    from sklearn.tree import DecisionTreeClassifier
    rng = np.random.default_rng(5)
    X = np.exp(rng.normal(3, 3, (500, O.NUM_FEATURES))).astype(np.float32)
    lab = (X[:, 3] > 20).astype(int) + 2 * (X[:, 6] > X[:, 3])
    clf = DecisionTreeClassifier(criterion="gini", max_depth=6, random_state=0).fit(X, lab)
    t = clf.tree_
    feat = np.where(t.children_left < 0, -1, t.feature)
    kl = clf.classes_[np.argmax(t.value[:, 0, :], axis=1)]
    tree = S.Tree(feat, t.threshold, t.children_left, t.children_right, kl)
    want = clf.predict(X)
    for r, w in zip(X, want):
        f = B.seer_features_t()
        for i in range(O.NUM_FEATURES):
            f.f[i] = float(r[i])
        assert S.seer_select(f, tree) == w


def test_malformed_trees_are_rejected():
    f = B.seer_features_t()
    bad = [
        S.Tree([0, -1, -1], [1.0, 0, 0], [1, -1, -1], [7, -1, -1], [-1, 0, 1]),     # child out of range
        S.Tree([0, 0], [1e30, 1e30], [1, 0], [1, 0], [0, 0]),                       # cycle
        S.Tree([13, -1, -1], [1.0, 0, 0], [1, -1, -1], [2, -1, -1], [-1, 0, 1]),    # feature index too large
        S.Tree([-1], [0.0], [-1], [-1], [S.NUM_KERNELS]),                           # class out of range
        S.Tree([0, -1, -1], [float("nan"), 0, 0], [1, -1, -1], [2, -1, -1], [-1, 0, 1]),
    ]
    for t in bad:
        with pytest.raises(S.SeerError) as ei:
            S.seer_select(f, t)
        assert ei.value.status == -3
    k = C.c_int(-7)
    assert S.lib().seer_select(None, C.byref(bad[0].c), C.byref(k)) == -1 and k.value == -7


def test_spmv_argument_errors_without_gpu():
    L = S.lib()
    A = B.seer_csr(0, 0, 0, None, None, None)
    assert L.seer_spmv(S.NUM_KERNELS, C.byref(A), None, None, None, 0, None) == -2
    assert L.seer_spmv(-1, C.byref(A), None, None, None, 0, None) == -2
    assert L.seer_spmv(0, None, None, None, None, 0, None) == -1
    assert L.seer_spmv(0, C.byref(A), None, None, None, 0, None) == -1          # row_ptr null
    dummy = (C.c_int32 * 4)()
    A = B.seer_csr(-1, 0, 0, C.cast(dummy, C.c_void_p), None, None)
    assert L.seer_spmv(0, C.byref(A), None, None, None, 0, None) == -1
    A = B.seer_csr(0, 5, 0, C.cast(dummy, C.c_void_p), None, None)
    assert L.seer_spmv(3, C.byref(A), None, None, None, 0, None) == 0           # rows == 0: nothing to do
    A = B.seer_csr(3, 5, 2, C.cast(dummy, C.c_void_p), None, None)
    assert L.seer_spmv(1, C.byref(A), None, None, None, 0, None) == -1          # nnz > 0 but no entries
    out = B.seer_features_t()
    assert L.seer_features(None, C.byref(out), None, 0, None) == -1
    A = B.seer_csr(3, 5, 2, C.cast(dummy, C.c_void_p), None, None)
    assert L.seer_features(C.byref(A), C.byref(out), None, 0, None) == -4       # no workspace
    A0 = B.seer_csr(0, 5, 0, C.cast(dummy, C.c_void_p), None, None)
    assert L.seer_features(C.byref(A0), C.byref(out), None, 0, None) == 0 and out.f[1] == 5.0


def test_overlapping_x_and_y_are_rejected_before_any_launch():
    """x [cols] and y [rows] must be disjoint; the check is pointer arithmetic on the host, so it
    can be exercised with host buffers standing in for device memory (nothing is launched)."""
    L = S.lib()
    ints = (C.c_int32 * 16)()
    buf = (C.c_float * 64)()
    base = C.addressof(buf)
    A = B.seer_csr(8, 8, 4, C.cast(ints, C.c_void_p), C.cast(ints, C.c_void_p), C.cast(buf, C.c_void_p))
    vp = C.c_void_p
    for kid in (S.CSR_TM, S.CSR_WM, S.CSR_BM):                      # no workspace needed before the check
        assert L.seer_spmv(kid, C.byref(A), vp(base), vp(base), None, 0, None) == -1            # the same vector
        assert L.seer_spmv(kid, C.byref(A), vp(base), vp(base + 4 * 7), None, 0, None) == -1    # y starts on x's last entry
        assert L.seer_spmv(kid, C.byref(A), vp(base + 4 * 7), vp(base), None, 0, None) == -1    # x starts on y's last entry
    t = S.Tree.constant(S.CSR_TM)
    assert L.seer_spmv_auto(C.byref(A), C.byref(t.c), vp(base), vp(base + 16), None, 0, None) == -1


def test_workspace_sizes():
    assert S.spmv_workspace_bytes(0, 10**6, 10**7) == 0
    assert S.spmv_workspace_bytes(2, 10**6, 10**7) == 0
    n_tiles = -(-(10**6 + 10**7) // (256 * 7))
    assert S.spmv_workspace_bytes(3, 10**6, 10**7) >= 8 * n_tiles
    assert S.features_workspace_bytes(10**6) >= 1024 * 32


def test_plan_argument_errors_and_sizes_without_gpu():
    """The preprocessing entry points reject bad arguments before any GPU work, and the
    size functions give what the header states."""
    L = S.lib()
    dummy = (C.c_int32 * 4)()
    A = B.seer_csr(3, 5, 2, C.cast(dummy, C.c_void_p), C.cast(dummy, C.c_void_p), C.cast(dummy, C.c_void_p))
    plan = B.seer_plan()
    assert L.seer_spmv_prepare(S.CSR_A, C.byref(A), None, 0, None, None) == -1            # no plan struct
    assert L.seer_spmv_prepare(S.NUM_KERNELS, C.byref(A), None, 0, None, C.byref(plan)) == -2
    assert L.seer_spmv_prepare(-1, C.byref(A), None, 0, None, C.byref(plan)) == -2
    assert L.seer_spmv_prepare(S.CSR_A, None, None, 0, None, C.byref(plan)) == -1
    assert L.seer_spmv_prepare(S.CSR_A, C.byref(A), None, 0, None, C.byref(plan)) == -4   # no plan memory
    assert L.seer_spmv_prepare(S.ELL_TM, C.byref(A), None, 0, None, C.byref(plan)) == -4
    # kernels without preprocessing: the call only records the id
    assert L.seer_spmv_prepare(S.CSR_BM, C.byref(A), None, 0, None, C.byref(plan)) == 0
    assert (plan.kernel_id, plan.rows, plan.nnz, plan.device) == (S.CSR_BM, 3, 2, None)
    assert L.seer_spmv_prepared_workspace_bytes(C.byref(plan)) == 0
    plan.kernel_id = S.CSR_MP
    assert L.seer_spmv_prepared_workspace_bytes(C.byref(plan)) == S.spmv_workspace_bytes(S.CSR_MP, 3, 2)
    assert L.seer_spmv_prepared_workspace_bytes(None) == 0
    assert L.seer_spmv_prepared(None, C.byref(A), None, None, None, 0, None) == -1
    # a CSR,A plan is tied to its matrix
    plan = B.seer_plan(S.CSR_A, 4, 2, 1, 0, 0, C.cast(dummy, C.c_void_p), 16)
    assert L.seer_spmv_prepared(C.byref(plan), C.byref(A), None, None, None, 0, None) == -1
    # selection for several products: argument checks
    t = S.Tree.constant(S.CSR_BM)
    model = S.Model(t)
    assert L.seer_spmv_plan(C.byref(A), C.byref(model.c), 0, None, 0, None, 0, None, C.byref(plan), None) == -1
    half = S.Model(t)
    half.c.selector = model.c.gathered                      # a selector without a known model
    assert L.seer_spmv_plan(C.byref(A), C.byref(half.c), 1, None, 0, None, 0, None, C.byref(plan), None) == -1
    # no model: the built-in one (generated code) decides; this tiny matrix needs neither features
    # nor preprocessing, so the call touches no device and only records its choice
    path = C.c_int(-1)
    before = bytes(plan)
    rc = L.seer_spmv_plan(C.byref(A), None, 1, None, 0, None, 0, None, C.byref(plan), C.byref(path))
    kf = S.seer_known_features(3, 5, 2)
    from paper_2403_17017_amd import training as T
    import os
    it_model, _ = T.load_model(os.path.join(os.path.dirname(T.__file__), "selector_model.json"), iterative=True)
    if S.seer_select(kf, it_model.selector) == 0 and S.seer_select(kf, it_model.known) < S.NUM_DIRECT_KERNELS:
        assert rc == 0 and path.value == 0
        assert plan.kernel_id == S.seer_select(kf, it_model.known) and bytes(plan) != before
    else:       # the shipped model wants features or a plan here: refused for want of memory, outputs untouched
        assert rc == -4 and path.value == -1 and bytes(plan) == before
    assert L.seer_spmv_plan(C.byref(A), C.byref(model.c), 1, None, 0, None, 0, None, None, None) == -1
    # sizes
    assert S.plan_bytes(S.CSR_BM, 10**6, 10**7) == 0 and S.plan_bytes(S.ELL_TM, 10**6, 10**7) == 0
    n_blocks = -(-10**7 // 2048)
    assert S.plan_bytes(S.CSR_A, 10**6, 10**7) >= 8 * (n_blocks + 1)
    assert S.plan_bytes(S.CSR_A, 10**6, 0) >= 16                                          # one block owns every row
    assert S.spmv_workspace_bytes(S.CSR_A, 10**6, 10**7) >= S.plan_bytes(S.CSR_A, 10**6, 10**7) + 8 * n_blocks
    # CSR,WO: one carry pair per chunk; chunks of 2048 nonzeros, of 4096 from 2^23 nonzeros on
    assert 8 * -(-10**7 // 4096) <= S.spmv_workspace_bytes(S.CSR_WO, 10**6, 10**7) < 8 * n_blocks
    assert S.spmv_workspace_bytes(S.CSR_WO, 10**6, 2**23 - 1) >= 8 * -(-(2**23 - 1) // 2048)
    assert S.plan_bytes(S.COO_WM, 10**6, 10**7) == 4 * 10**7 + (-4 * 10**7) % 256
    assert S.spmv_workspace_bytes(S.COO_WM, 10**6, 10**7) >= S.plan_bytes(S.COO_WM, 10**6, 10**7) + 8 * -(-10**7 // 512)
    assert S.ell_plan_bytes(1000, 5) == 2 * 1024 * 5 * 4
    assert S.ell_plan_bytes(1000, 0) > 0 and S.ell_plan_bytes(0, 5) == 0
    assert S.ell_plan_bytes(2**20, 2**11) == 0 and S.ell_plan_bytes(2**20, 2**11 - 1) > 0   # 2^31 slots: not applicable


def test_trees_for_the_single_product_paths_must_name_direct_kernels():
    """seer_spmv_auto / seer_spmv_model reject, before any GPU work, a tree whose leaf names a
    kernel that needs preprocessing."""
    L = S.lib()
    dummy = (C.c_int32 * 4)()
    A = B.seer_csr(3, 5, 2, C.cast(dummy, C.c_void_p), C.cast(dummy, C.c_void_p), C.cast(dummy, C.c_void_p))
    for kid in (S.CSR_A, S.ELL_TM, S.COO_WM):
        t = S.Tree.constant(kid)
        assert L.seer_spmv_auto(C.byref(A), C.byref(t.c), None, None, None, 0, None) == -3
        never_gather = S.Tree([-1], [0.0], [-1], [-1], [0], n_classes=2)
        model = S.Model(S.Tree.constant(S.CSR_BM), t, never_gather)
        assert L.seer_spmv_model(C.byref(A), C.byref(model.c), None, None, None, 0, None, None, None) == -3


C_CLIENT = r"""
#include "seer.h"
#include <stdio.h>
#include <string.h>

/* every entry point of the header, by address: the prototypes are plain C */
typedef void (*any_fn)(void);
static const any_fn entry_points[] = {
    (any_fn)seer_features, (any_fn)seer_features_workspace_bytes, (any_fn)seer_derive_features,
    (any_fn)seer_known_features, (any_fn)seer_select, (any_fn)seer_spmv, (any_fn)seer_spmv_workspace_bytes,
    (any_fn)seer_spmv_auto, (any_fn)seer_spmv_auto_workspace_bytes, (any_fn)seer_spmv_model,
    (any_fn)seer_spmv_auto_result, (any_fn)seer_plan_bytes, (any_fn)seer_ell_plan_bytes, (any_fn)seer_spmv_prepare,
    (any_fn)seer_spmv_prepared, (any_fn)seer_spmv_prepared_workspace_bytes, (any_fn)seer_spmv_plan,
    (any_fn)seer_csr_check, (any_fn)seer_set_tuning, (any_fn)seer_stream_copy, (any_fn)seer_stream_sum,
    (any_fn)seer_gather_sum, (any_fn)seer_num_kernels, (any_fn)seer_kernel_name, (any_fn)seer_strerror,
    (any_fn)seer_last_hip_error};

int main(void)
{
    seer_features_t f;
    seer_node nodes[3] = {{SEER_F_MEAN_LEN, 1, 2, -1, 8.0}, {-1, -1, -1, SEER_CSR_TM, 0.0}, {-1, -1, -1, SEER_CSR_WO, 0.0}};
    seer_tree tree = {3, SEER_NUM_FEATURES, SEER_NUM_KERNELS, nodes};
    int kid = -1, rc, i;
    for (i = 0; i < (int)(sizeof entry_points / sizeof entry_points[0]); ++i)
        if (!entry_points[i]) return 2;
    memset(&f, 0, sizeof f);
    f.rows = 4; f.cols = 20; f.nnz = 20; f.max_len = 5; f.min_len = 5; f.empty_rows = 0; f.sum_sq_len = 100;
    rc = seer_derive_features(&f);                      /* four rows of 5 nonzeros in 20 columns */
    printf("derive %d mean %.6f density %.6f var %.6f\n", rc, f.f[SEER_F_MEAN_LEN], f.f[SEER_F_MEAN_DENSITY], f.f[SEER_F_VAR_LEN]);
    rc = seer_select(&f, &tree, &kid);
    printf("select %d kernel %d %s\n", rc, kid, seer_kernel_name(kid));
    f.f[SEER_F_MEAN_LEN] = 9.0f;
    rc = seer_select(&f, &tree, &kid);
    printf("select %d kernel %d %s\n", rc, kid, seer_kernel_name(kid));
    printf("kernels %d workspace %lu error \"%s\"\n", seer_num_kernels(),
           (unsigned long)seer_spmv_workspace_bytes(SEER_CSR_TM, 1000, 5000), seer_strerror(SEER_ETREE));
    printf("null matrix %d\n", seer_spmv(SEER_CSR_TM, NULL, NULL, NULL, NULL, 0, NULL));
    return 0;
}
"""


def test_plain_c_client_compiles_against_the_header_and_runs(tmp_path):
    """The boundary is a C ABI: a C99 translation unit that includes only seer.h compiles
    without warnings, links against the library and gets the host-side answers (no GPU call).
    The density is the one of the paper's worked example (Sec. IV-A): 5 nonzeros in a row of
    20 columns -> 0.25."""
    import subprocess
    from paper_2403_17017_amd import binding
    S.lib()                                              # make sure the library is built
    src = tmp_path / "client.c"
    src.write_text(C_CLIENT)
    exe = tmp_path / "client"
    libdir = os.path.dirname(binding.LIB_PATH)
    include = os.path.join(os.path.dirname(libdir), "include")
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", include, "-o", str(exe),
                           str(src), binding.LIB_PATH, f"-Wl,-rpath,{libdir}", "-Wl,-rpath-link,/opt/rocm/lib",
                           "-Wl,--allow-shlib-undefined"])
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stderr
    lines = out.stdout.strip().splitlines()
    assert lines[0] == "derive 0 mean 5.000000 density 0.250000 var 0.000000"
    assert lines[1] == "select 0 kernel 0 CSR,TM"
    assert lines[2] == "select 0 kernel 4 CSR,WO"
    assert lines[3] == 'kernels 9 workspace 0 error "%s"' % S.strerror(-3)
    assert lines[4] == "null matrix -1"
