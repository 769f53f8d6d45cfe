"""GPU parity: every SpMV schedule, the feature reduction and the selector, called
through the C ABI, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import paper_2403_17017_amd as S
from oracle import seer_oracle as O
from workloads import csr_gen as G

from gpu_util import (announce, assert_features_equal, assert_parity, oracle_of, run_spmv, upload)

pytestmark = pytest.mark.gpu
KERNELS = [0, 1, 2, 3, 4, 5, 7]     # every id seer_spmv accepts (ELL,TM has no one-call form)


def edge_cases():
    c = []
    c.append(G.explicit_lengths([0, 0, 0], 4, 2, "all-empty"))
    c.append(G.explicit_lengths([1], 1, 3, "1x1"))
    c.append(G.explicit_lengths([0, 7, 0, 0, 3, 0], 7, 4, "empties+full-row"))
    c.append(G.explicit_lengths([64] + [0] * 10, 64, 5, "one-full-row"))
    c.append(G.explicit_lengths([9] * 6, 3, 6, "duplicate-columns"))
    c.append(G.explicit_lengths([0] * 5000 + [300_000] + [0] * 5000, 70_000, 7, "giant-row-among-empties"))
    c.append(G.explicit_lengths([100_003], 50_000, 8, "single-row-100k"))
    c.append(G.explicit_lengths([0] * 199_990 + [1] * 10, 1000, 9, "rows>>nnz"))
    c.append(G.explicit_lengths([6] * (256 * 9 + 17), 500, 10, "len6: 7 merge items per row"))
    c.append(G.explicit_lengths([14] * (256 * 5 + 3), 500, 11, "len14: 15 merge items per row"))
    c.append(G.explicit_lengths([1791] + [0] + [1792] * 3 + [5, 0, 0, 3839, 3840, 1], 4000, 12, "tile-sized rows"))
    c.append(G.explicit_lengths([2048, 2047, 2049, 1, 4096, 0, 33, 32, 31], 5000, 13, "chunk-sized rows"))
    c.append(G.explicit_lengths([0, 0, 0, 4097, 0, 2048, 2048, 1, 0, 6143, 2, 2046, 0, 0], 3000, 14, "blocks inside rows"))
    c.append(G.explicit_lengths([2048] * 7 + [1024] * 6 + [4096] * 3 + [0] * 1500, 2500, 15, "rows on block boundaries"))
    # rows cut into 4 ... 141 chunks / merge tiles: carry runs around the fix-up's boundaries
    # (partials fetched at once by the run's head; 64 per trip of the head's wave)
    c.append(G.explicit_lengths([2048 * 4 + 100, 3, 2048 * 5 + 100, 0, 2048 * 6 + 7, 1, 2048 * 68 + 5, 2,
                                 2048 * 69 + 9, 2048 * 70 + 1, 5, 2048 * 140 + 77, 1], 300_000, 16, "carry runs"))
    return c


def medium_cases():
    c = []
    c.append(G.fixed_degree(4096, 4096, 16))                       # BASELINE config 1 at full size
    c.append(G.random_lengths(5003, 3000, 0, 40, 21))
    c.append(G.random_lengths(1237, 9000, 50, 700, 22))
    c.append(G.zipf_rows(20_011, s=1.6, cap=5000, seed=23))
    c.append(G.zipf_rows(60_000, s=1.3, cap=60_000, seed=24))
    c.append(G.laplacian_5pt(100))
    c.append(G.empty_poisson(100_003, 20_000, 0.3, 4.0, seed=25))
    c.append(G.banded(30_001, 9, 26))
    return c


ALL = edge_cases() + medium_cases()


@pytest.fixture(scope="module")
def cases():
    out = []
    for A in ALL:
        A.validate()
        x = G.dense_vector(A.cols, 1000 + len(out))
        y_ref, bound = oracle_of(A, x)
        out.append((A, x, y_ref, bound))
    return out


@pytest.mark.parametrize("kid", KERNELS)
def test_spmv_parity_default_launch(cases, kid):
    import torch
    for A, x, y_ref, bound in cases:
        announce(f"spmv kernel={kid} default launch, {A.name} rows={A.rows} nnz={A.nnz}")
        dA = upload(A)
        y = run_spmv(kid, dA, torch.from_numpy(x).cuda(), A.rows)
        assert_parity(y, y_ref, bound, f"kernel {kid} on {A.name}")


@pytest.mark.parametrize("knob,values,kid", [
    ("wm_lanes", [2, 4, 8, 16, 32, 64], 1),
    ("bm_rows", [1, 3, 7, 16, 17, 64, 100, 1024, 2048], 2),
    ("bm_chunk", [2048, 4096], 2),
    ("mp_ipt", [7, 15], 3),
])
def test_spmv_parity_every_launch_shape(cases, knob, values, kid):
    import torch
    try:
        for v in values:
            S.set_tuning(knob, v)
            for remap in (0, 1):
                S.set_tuning("xcd_remap", remap)
                for A, x, y_ref, bound in cases:
                    if knob == "bm_rows" and v < 64 and A.rows > 50_000:
                        continue   # tiny blocks on big matrices only cost time
                    announce(f"spmv kernel={kid} {knob}={v} remap={remap}, {A.name}")
                    y = run_spmv(kid, upload(A), torch.from_numpy(x).cuda(), A.rows)
                    assert_parity(y, y_ref, bound, f"kernel {kid} {knob}={v} remap={remap} on {A.name}")
    finally:
        S.set_tuning(knob, -1)
        S.set_tuning("xcd_remap", -1)


@pytest.mark.parametrize("kid", KERNELS)
def test_spmv_parity_tile_orders_and_load_hints(cases, kid):
    """Every kernel under the round-robin tile order and with plain instead of streaming
    loads (the defaults are the XCD-contiguous order and the streaming hint)."""
    import torch
    try:
        for remap, nt in ((0, 0), (0, 1), (1, 0)):
            S.set_tuning("xcd_remap", remap)
            S.set_tuning("nt", nt)
            for A, x, y_ref, bound in cases:
                announce(f"spmv kernel={kid} remap={remap} nt={nt}, {A.name}")
                y = run_spmv(kid, upload(A), torch.from_numpy(x).cuda(), A.rows)
                assert_parity(y, y_ref, bound, f"kernel {kid} remap={remap} nt={nt} on {A.name}")
    finally:
        S.set_tuning("xcd_remap", -1)
        S.set_tuning("nt", -1)


@pytest.mark.parametrize("runs", [0, 1])
def test_coo_both_forms_on_every_case(cases, runs):
    """COO,WM sums an interval in one of two ways (a tuning switch picks); each
    forced onto every case, also with entry arrays off a 16-byte boundary, and with integer
    data, where the two forms and the oracle must agree to the bit."""
    import torch
    try:
        S.set_tuning("coo_runs", runs)
        for A, x, y_ref, bound in cases:
            for mis in (False, True):
                if mis and A.nnz == 0:
                    continue
                announce(f"COO,WM runs={runs} misaligned={mis}, {A.name}")
                y = run_spmv(S.COO_WM, upload(A, misalign=mis), torch.from_numpy(x).cuda(), A.rows)
                assert_parity(y, y_ref, bound, f"COO,WM runs={runs} misaligned={mis} on {A.name}")
            Ai = G.small_integer_values(A, seed=91)
            xi = np.random.default_rng(92).integers(-3, 4, A.cols).astype(np.float32)
            yi_ref, bi = oracle_of(Ai, xi)
            if A.nnz and float(bi.max()) >= 2.0**24:
                continue
            yi = run_spmv(S.COO_WM, upload(Ai), torch.from_numpy(xi).cuda(), A.rows)
            assert np.array_equal(yi, yi_ref.astype(np.float32)), f"COO,WM runs={runs}: integer data not exact on {A.name}"
    finally:
        S.set_tuning("coo_runs", -1)


@pytest.mark.parametrize("kid", KERNELS)
def test_spmv_misaligned_entries(cases, kid):
    import torch
    for A, x, y_ref, bound in cases:
        if A.nnz == 0:
            continue
        announce(f"spmv kernel={kid} misaligned col/val, {A.name}")
        y = run_spmv(kid, upload(A, misalign=True), torch.from_numpy(x).cuda(), A.rows)
        assert_parity(y, y_ref, bound, f"kernel {kid} misaligned on {A.name}")


@pytest.mark.parametrize("kid", KERNELS)
def test_spmv_bit_exact_cases(kid):
    """Results that do not depend on summation order must match the oracle exactly."""
    import torch
    rng = np.random.default_rng(77)
    # (a) at most one nonzero per row: y_i = fl32(a_i * x_c), a single correctly rounded product
    n = 70_001
    lens = (rng.random(n) < 0.8).astype(np.int64)
    A = G.explicit_lengths(lens, 5000, 78, "<=1 per row")
    x = G.dense_vector(A.cols, 79)
    y_ref, _ = oracle_of(A, x)
    announce(f"bit-exact kernel={kid} {A.name}")
    y = run_spmv(kid, upload(A), torch.from_numpy(x).cuda(), A.rows)
    assert np.array_equal(y, y_ref.astype(np.float32))
    # identity: y == x
    I = G.HostCSR(n, n, np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32), np.ones(n, np.float32), "I")
    xi = G.dense_vector(n, 80)
    y = run_spmv(kid, upload(I), torch.from_numpy(xi).cuda(), n)
    assert np.array_equal(y, xi)
    # (b) small integers everywhere: every partial sum is an exact fp32 integer
    for B in (G.zipf_rows(30_000, s=1.5, cap=20_000, seed=81), G.random_lengths(9000, 4000, 0, 60, 82)):
        Bi = G.small_integer_values(B, 83)
        xb = np.round(G.dense_vector(Bi.cols, 84) * 4).astype(np.float32)
        y_ref, _ = oracle_of(Bi, xb)
        announce(f"bit-exact kernel={kid} integer values {Bi.name}")
        y = run_spmv(kid, upload(Bi), torch.from_numpy(xb).cuda(), Bi.rows)
        assert np.array_equal(y.astype(np.float64), y_ref)
    # x = 1: row sums
    Bi = G.small_integer_values(G.empty_poisson(50_000, 9000, 0.3, 4.0, seed=85), 86)
    y_ref, _ = oracle_of(Bi, np.ones(Bi.cols, np.float32))
    y = run_spmv(kid, upload(Bi), torch.ones(Bi.cols, device="cuda:0"), Bi.rows)
    assert np.array_equal(y.astype(np.float64), y_ref)


@pytest.mark.parametrize("kid", KERNELS)
def test_spmv_deterministic_and_no_prezero_needed(cases, kid):
    import torch
    A, x, y_ref, bound = next(c for c in cases if c[0].name.startswith("zipf1.6_20011"))
    dA = upload(A)
    xd = torch.from_numpy(x).cuda()
    announce(f"determinism kernel={kid} {A.name}")
    y1 = run_spmv(kid, dA, xd, A.rows, poison=True)
    y2 = run_spmv(kid, dA, xd, A.rows, poison=False)
    y3 = run_spmv(kid, dA, xd, A.rows, poison=True)
    assert y1.tobytes() == y2.tobytes() == y3.tobytes()


def test_rows_zero_and_status_codes():
    import torch
    A = G.explicit_lengths([], 5, 1, "0x5")
    dA = upload(A)
    y = torch.full((4,), 7.0, device="cuda:0")
    for kid in KERNELS:
        S.seer_spmv(kid, dA, torch.zeros(5, device="cuda:0"), y)
    torch.cuda.synchronize()
    assert torch.all(y == 7.0)
    B = G.random_lengths(100, 50, 0, 5, 3)
    dB = upload(B)
    with pytest.raises(S.SeerError) as ei:
        S.seer_spmv(S.ELL_TM, dB, torch.zeros(50, device="cuda:0"), torch.zeros(100, device="cuda:0"))
    assert ei.value.status == -2          # no one-call form: its plan size depends on the matrix
    with pytest.raises(S.SeerError) as ei:
        S.seer_spmv(S.NUM_KERNELS, dB, torch.zeros(50, device="cuda:0"), torch.zeros(100, device="cuda:0"))
    assert ei.value.status == -2
    small = torch.empty(16, dtype=torch.uint8, device="cuda:0")
    big = G.random_lengths(100_000, 50, 0, 5, 3)
    for kid in (S.CSR_MP, S.CSR_WO):
        with pytest.raises(S.SeerError) as ei:
            S.seer_spmv(kid, upload(big), torch.zeros(50, device="cuda:0"), torch.zeros(100_000, device="cuda:0"),
                        workspace=small)
        assert ei.value.status == -4


# ------------------------------------------------------------------ features + select
def test_features_bit_exact(cases):
    ws = S.alloc_workspace(S.features_workspace_bytes(1))
    for A, *_ in cases + [(G.explicit_lengths([], 5, 1, "0x5"),)]:
        announce(f"features {A.name} rows={A.rows}")
        got = S.seer_features(upload(A), workspace=ws)
        assert_features_equal(got, O.features(A.rows, A.cols, A.row_ptr), A.name)


def test_features_repeated_calls_reuse_workspace():
    """Back-to-back reductions of different sizes through one workspace (one workgroup,
    many partials, the cap on partials): nothing left by one call may leak into the next."""
    mats = [G.random_lengths(r, 1000, 0, 9, 300 + i) for i, r in enumerate([1, 4096, 4097, 70_000, 5_000_000, 17])]
    dev = [upload(A) for A in mats]
    want = [O.features(A.rows, A.cols, A.row_ptr) for A in mats]
    ws = S.alloc_workspace(S.features_workspace_bytes(1))
    for rep in range(25):
        for A, d, w in zip(mats, dev, want):
            if rep == 0:
                announce(f"features repeat {A.name}")
            assert_features_equal(S.seer_features(d, workspace=ws), w, f"{A.name} rep {rep}")


def test_select_end_to_end_matches_oracle(cases):
    from sklearn.tree import DecisionTreeClassifier
    feats = np.stack([O.features(A.rows, A.cols, A.row_ptr)["f"] for A, *_ in cases])
    lab = np.arange(len(cases)) % 4
    clf = DecisionTreeClassifier(criterion="gini", max_depth=6, random_state=0).fit(feats, lab)
    t = clf.tree_
    feat = np.where(t.children_left < 0, -1, t.feature)
    kl = clf.classes_[np.argmax(t.value[:, 0, :], axis=1)]
    tree = S.Tree(feat, t.threshold, t.children_left, t.children_right, kl)
    import torch
    for (A, x, y_ref, bound), f_or in zip(cases, feats):
        d = upload(A)
        f = S.seer_features(d)
        kid = S.seer_select(f, tree)
        assert kid == O.select(f_or, *tree.arrays) == int(clf.predict(f_or[None])[0])
        y = run_spmv(kid, d, torch.from_numpy(x).cuda(), A.rows)
        assert_parity(y, y_ref, bound, f"selected kernel {kid} on {A.name}")
