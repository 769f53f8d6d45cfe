"""GPU parity of the preprocessing split (seer_spmv_prepare / seer_spmv_prepared /
seer_spmv_plan): the plan the device writes must equal the oracle's plan entry for
entry, the product with it must match the oracle, and selection with an iteration count
must match the oracle's inference."""
import numpy as np
import pytest

import paper_2403_17017_amd as S
from oracle import seer_oracle as O
from workloads import csr_gen as G

from gpu_util import announce, assert_parity, oracle_of, run_spmv, upload
from test_gpu_parity import ALL

pytestmark = pytest.mark.gpu
CHUNK = 2048   # nonzeros per row block of CSR,A, as stated at seer_spmv_prepare


@pytest.fixture(scope="module")
def cases():
    out = []
    for A in ALL + [G.zipf_rows(200_000, s=1.4, cap=150_000, seed=31)]:
        x = G.dense_vector(A.cols, 3000 + len(out))
        y_ref, bound = oracle_of(A, x)
        out.append((A, x, y_ref, bound))
    return out


def test_plan_entries_bit_exact(cases):
    seen_split = set()
    for A, *_ in cases:
        announce(f"plan entries {A.name} rows={A.rows} nnz={A.nnz}")
        plan = S.seer_spmv_prepare(S.CSR_A, upload(A))
        row, start = O.adaptive_plan(A.rows, A.row_ptr, CHUNK)
        assert plan.kernel_id == S.CSR_A and plan.n_blocks == len(row) - 1
        got = plan.entries().astype(np.int64)
        assert np.array_equal(got[:, 0], row), f"first rows differ on {A.name}"
        assert np.array_equal(got[:, 1], start), f"first nonzeros differ on {A.name}"
        split = bool(np.any(row[1:] == row[:-1]))
        assert plan.split_rows == split, A.name
        carries = 2 * ((4 * plan.n_blocks + 255) // 256 * 256)      # one (row, partial) pair per block, if any row is split
        assert S.spmv_prepared_workspace_bytes(plan) == (carries if split else 0)
        seen_split.add(split)
    assert seen_split == {True, False}


def test_prepared_product_parity_and_reuse(cases):
    import torch
    for A, x, y_ref, bound in cases:
        announce(f"prepared product {A.name}")
        dA = upload(A)
        xd = torch.from_numpy(x).cuda()
        plan = S.seer_spmv_prepare(S.CSR_A, dA)
        single = run_spmv(S.CSR_A, dA, xd, A.rows)
        for rep in range(3):      # the plan is read-only: every product gives the same bits
            y = torch.full((max(A.rows, 1),), float("nan"), device="cuda:0")
            S.seer_spmv_prepared(plan, dA, xd, y)
            torch.cuda.synchronize()
            got = y[:A.rows].cpu().numpy()
            assert_parity(got, y_ref, bound, f"prepared CSR,A on {A.name}")
            assert got.tobytes() == single.tobytes(), f"prepared and single-call CSR,A differ on {A.name}"


def test_prepared_misaligned_entries(cases):
    import torch
    for A, x, y_ref, bound in cases:
        if A.nnz == 0:
            continue
        announce(f"prepared product, misaligned entries, {A.name}")
        dA = upload(A, misalign=True)
        plan = S.seer_spmv_prepare(S.CSR_A, dA)
        y = torch.full((A.rows,), float("nan"), device="cuda:0")
        S.seer_spmv_prepared(plan, dA, torch.from_numpy(x).cuda(), y)
        assert_parity(y.cpu().numpy(), y_ref, bound, f"prepared CSR,A misaligned on {A.name}")


def test_prepared_in_a_hip_graph(cases):
    import torch
    picks = [c for c in cases if c[0].name.startswith(("zipf1.6_20011", "laplace5_100", "blocks inside rows"))]
    assert len(picks) == 3
    for A, x, y_ref, bound in picks:
        dA, xd = upload(A), torch.from_numpy(x).cuda()
        plan = S.seer_spmv_prepare(S.CSR_A, dA)
        ws = S.alloc_workspace(S.spmv_prepared_workspace_bytes(plan))
        y = torch.full((A.rows,), float("nan"), device="cuda:0")
        S.seer_spmv_prepared(plan, dA, xd, y, ws)
        torch.cuda.synchronize()
        eager = y.clone()
        announce(f"prepared product graph capture {A.name}")
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            S.seer_spmv_prepared(plan, dA, xd, y, ws)
        for rep in range(4):
            y.fill_(float("nan"))                        # eager work between replays
            _ = run_spmv(S.CSR_MP, dA, xd, A.rows)
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(y, eager), f"replay {rep} differs on {A.name}"
        assert_parity(y.cpu().numpy(), y_ref, bound, f"prepared graph replay on {A.name}")


def test_kernels_without_preprocessing_prepare_to_themselves(cases):
    import torch
    A, x, y_ref, bound = next(c for c in cases if c[0].name.startswith("zipf1.6_20011"))
    dA, xd = upload(A), torch.from_numpy(x).cuda()
    for kid in range(S.NUM_DIRECT_KERNELS):
        assert S.plan_bytes(kid, A.rows, A.nnz) == 0
        plan = S.seer_spmv_prepare(kid, dA)
        assert plan.kernel_id == kid and plan.c.device is None
        y = torch.full((A.rows,), float("nan"), device="cuda:0")
        S.seer_spmv_prepared(plan, dA, xd, y)
        torch.cuda.synchronize()
        assert y.cpu().numpy().tobytes() == run_spmv(kid, dA, xd, A.rows).tobytes()


def test_plan_status_codes():
    import torch
    A = G.random_lengths(3000, 500, 0, 9, 3)
    B = G.random_lengths(3001, 500, 0, 9, 4)
    dA, dB = upload(A), upload(B)
    with pytest.raises(S.SeerError) as ei:
        S.seer_spmv_prepare(S.CSR_A, dA, plan_mem=torch.empty(16, dtype=torch.uint8, device="cuda:0"))
    assert ei.value.status == -4
    with pytest.raises(S.SeerError) as ei:
        S.seer_spmv_prepare(S.NUM_KERNELS, dA)
    assert ei.value.status == -2
    plan = S.seer_spmv_prepare(S.CSR_A, dA)
    x, y = torch.zeros(500, device="cuda:0"), torch.zeros(3001, device="cuda:0")
    with pytest.raises(S.SeerError) as ei:
        S.seer_spmv_prepared(plan, dB, x, y)          # a plan belongs to one matrix
    assert ei.value.status == -1
    long_row = upload(G.explicit_lengths([10_000], 100, 5, "one long row"))
    plan = S.seer_spmv_prepare(S.CSR_A, long_row)
    assert plan.split_rows
    with pytest.raises(S.SeerError) as ei:
        S.seer_spmv_prepared(plan, long_row, x, y, workspace=torch.empty(16, dtype=torch.uint8, device="cuda:0"))
    assert ei.value.status == -4
    empty = upload(G.explicit_lengths([], 5, 1, "0x5"))
    plan = S.seer_spmv_prepare(S.CSR_A, empty)
    S.seer_spmv_prepared(plan, empty, x, y)            # rows == 0: nothing to do, no error


def test_selection_with_an_iteration_count(cases):
    """seer_spmv_plan: both paths, both sides of an iteration threshold, against the
    oracle's inference; then the products with the plan it returns."""
    import torch
    # selector: rows <= 50000 -> known model, else gather
    selector = S.Tree([0, -1, -1], [50000.0, 0, 0], [1, -1, -1], [2, -1, -1], [-1, 0, 1], n_classes=2)
    # known: iterations <= 18.5 ? CSR,BM : CSR,A
    known = S.Tree([12, -1, -1], [18.5, 0, 0], [1, -1, -1], [2, -1, -1], [-1, 2, 5])
    # gathered: var_len <= 50 ? (iterations <= 3.5 ? CSR,TM : CSR,A) : (iterations <= 7.5 ? CSR,MP : CSR,A)
    gathered = S.Tree([6, 12, 12, -1, -1, -1, -1], [50.0, 3.5, 7.5, 0, 0, 0, 0], [1, 3, 5, -1, -1, -1, -1],
                      [2, 4, 6, -1, -1, -1, -1], [-1, -1, -1, 0, 5, 3, 5])
    model = S.Model(gathered, known, selector)
    seen = set()
    for A, x, y_ref, bound in cases:
        dA, xd = upload(A), torch.from_numpy(x).cuda()
        for iterations in (1, 4, 8, 19):
            announce(f"selection for {iterations} iterations, {A.name}")
            plan, path = S.seer_spmv_plan(dA, model, iterations)
            fg = O.features(A.rows, A.cols, A.row_ptr, iterations)["f"]
            want = O.model_select(A.rows, A.cols, A.nnz, fg, selector.arrays, known.arrays, gathered.arrays,
                                  iterations)
            assert (path, plan.kernel_id) == want, (A.name, iterations)
            seen.add(want)
            y = torch.full((max(A.rows, 1),), float("nan"), device="cuda:0")
            for _ in range(2):
                S.seer_spmv_prepared(plan, dA, xd, y)
            torch.cuda.synchronize()
            assert_parity(y[:A.rows].cpu().numpy(), y_ref, bound, f"planned kernel {plan.kernel_id} on {A.name}")
    assert {(0, 2), (0, 5), (1, 0), (1, 3), (1, 5)} <= seen


# ------------------------------------------------------------------ ELL,TM
def ell_cases(cases):
    """Matrices whose ELL form is of reasonable size (longest row * rows <= 16 M slots)."""
    return [c for c in cases if c[0].rows > 0 and int(np.diff(c[0].row_ptr).max(initial=0)) * c[0].rows <= 16_000_000]


def test_ell_arrays_bit_exact(cases):
    picks = ell_cases(cases)
    assert len(picks) >= 12
    for A, *_ in picks:
        announce(f"ELL conversion {A.name} rows={A.rows} nnz={A.nnz}")
        plan = S.seer_spmv_prepare(S.ELL_TM, upload(A))
        want_c, want_v = O.ell_from_csr(A.rows, A.row_ptr, A.col_idx, A.values)
        assert plan.kernel_id == S.ELL_TM and plan.ell_width == want_c.shape[0]
        got_c, got_v = plan.ell_arrays()
        assert np.array_equal(got_c, want_c), f"ELL columns differ on {A.name}"
        assert got_v.tobytes() == want_v.tobytes(), f"ELL values differ on {A.name}"
        assert S.spmv_prepared_workspace_bytes(plan) == 0


def test_ell_product_parity(cases):
    import torch
    for A, x, y_ref, bound in ell_cases(cases):
        announce(f"ELL,TM product {A.name}")
        for mis in (False, True):
            if mis and A.nnz == 0:
                continue
            dA = upload(A, misalign=mis)
            plan = S.seer_spmv_prepare(S.ELL_TM, dA)
            xd = torch.from_numpy(x).cuda()
            first = None
            for rep in range(2):
                y = torch.full((A.rows,), float("nan"), device="cuda:0")
                S.seer_spmv_prepared(plan, dA, xd, y)
                torch.cuda.synchronize()
                got = y.cpu().numpy()
                assert_parity(got, y_ref, bound, f"ELL,TM on {A.name}")
                first = got if first is None else first
                assert got.tobytes() == first.tobytes()


def test_ell_padding_is_inert_and_exact_cases():
    """An infinite x entry must reach only the rows that hold its column (a padded slot that
    multiplied 0 * inf would give NaN); integer data gives the exact row sums."""
    import torch
    A = G.small_integer_values(G.random_lengths(5000, 300, 0, 9, 41), 42)
    x = np.round(G.dense_vector(A.cols, 43) * 4).astype(np.float32)
    dA = upload(A)
    plan = S.seer_spmv_prepare(S.ELL_TM, dA)
    y = torch.empty(A.rows, device="cuda:0")
    S.seer_spmv_prepared(plan, dA, torch.from_numpy(x).cuda(), y)
    y_ref, _ = oracle_of(A, x)
    assert np.array_equal(y.cpu().numpy().astype(np.float64), y_ref)
    x[0] = np.inf
    S.seer_spmv_prepared(plan, dA, torch.from_numpy(x).cuda(), y)
    got = y.cpu().numpy()
    has0 = np.array([0 in A.col_idx[A.row_ptr[i]:A.row_ptr[i + 1]] for i in range(A.rows)])
    assert not np.any(np.isnan(got[~has0])) and np.all(np.isfinite(got[~has0]))
    assert np.all(~np.isfinite(got[has0]))


def test_ell_in_a_hip_graph_and_status_codes(cases):
    import torch
    A, x, y_ref, bound = next(c for c in cases if c[0].name.startswith("laplace5_100"))
    dA, xd = upload(A), torch.from_numpy(x).cuda()
    plan = S.seer_spmv_prepare(S.ELL_TM, dA)
    y = torch.full((A.rows,), float("nan"), device="cuda:0")
    S.seer_spmv_prepared(plan, dA, xd, y)
    torch.cuda.synchronize()
    eager = y.clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        S.seer_spmv_prepared(plan, dA, xd, y)
    for rep in range(3):
        y.fill_(float("nan"))
        _ = run_spmv(S.CSR_BM, dA, xd, A.rows)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, eager)
    assert_parity(y.cpu().numpy(), y_ref, bound, "ELL,TM graph replay")
    # plan memory too small: the call says how much it needs
    small = torch.empty(S.features_workspace_bytes(A.rows), dtype=torch.uint8, device="cuda:0")
    with pytest.raises(S.SeerError) as ei:
        S.seer_spmv_prepare(S.ELL_TM, dA, plan_mem=small)
    assert ei.value.status == -4
    assert S.ell_plan_bytes(A.rows, 5) == 2 * (-(-A.rows // 64) * 64) * 5 * 4
    # a row so long that the padded arrays cannot be indexed: not applicable
    assert S.ell_plan_bytes(2_000_000, 200_000) == 0
    giant = upload(G.explicit_lengths([0] * 50_000 + [70_000] + [0] * 50_000, 70_000, 7, "giant row"))
    with pytest.raises(S.SeerError) as ei:
        S.seer_spmv_prepare(S.ELL_TM, giant, plan_mem=torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0"))
    assert ei.value.status == -1


def test_plan_falls_back_to_adaptive_when_ell_does_not_fit(cases):
    import torch
    always_ell = S.Tree.constant(S.ELL_TM)
    model = S.Model(always_ell, always_ell, S.Tree([-1], [0.0], [-1], [-1], [1], n_classes=2))
    for name, want in (("laplace5_100", S.ELL_TM), ("giant-row-among-empties", S.CSR_A)):
        A, x, y_ref, bound = next(c for c in cases if c[0].name.startswith(name))
        dA, xd = upload(A), torch.from_numpy(x).cuda()
        plan_mem = S.alloc_workspace(max(S.plan_bytes(S.CSR_A, A.rows, A.nnz), 1 << 20))
        plan, path = S.seer_spmv_plan(dA, model, 50, plan_mem=plan_mem)
        assert path == 1 and plan.kernel_id == want, name
        y = torch.full((A.rows,), float("nan"), device="cuda:0")
        S.seer_spmv_prepared(plan, dA, xd, y)
        assert_parity(y.cpu().numpy(), y_ref, bound, f"planned {S.kernel_name(plan.kernel_id)} on {name}")


# ------------------------------------------------------------------ COO,WM
def test_coo_rows_bit_exact_and_product_parity(cases):
    import torch
    for A, x, y_ref, bound in cases:
        announce(f"COO,WM conversion and product {A.name} rows={A.rows} nnz={A.nnz}")
        dA = upload(A)
        plan = S.seer_spmv_prepare(S.COO_WM, dA)
        assert plan.kernel_id == S.COO_WM
        assert np.array_equal(plan.coo_rows(), O.coo_rows_from_csr(A.rows, A.row_ptr)), f"row indices differ on {A.name}"
        xd = torch.from_numpy(x).cuda()
        single = run_spmv(S.COO_WM, dA, xd, A.rows)
        for rep in range(2):
            y = torch.full((max(A.rows, 1),), float("nan"), device="cuda:0")   # every row must be written, empty ones too
            S.seer_spmv_prepared(plan, dA, xd, y)
            torch.cuda.synchronize()
            got = y[:A.rows].cpu().numpy()
            assert_parity(got, y_ref, bound, f"COO,WM on {A.name}")
            assert got.tobytes() == single.tobytes()
        if A.nnz:
            dM = upload(A, misalign=True)
            y = torch.full((A.rows,), float("nan"), device="cuda:0")
            S.seer_spmv_prepared(S.seer_spmv_prepare(S.COO_WM, dM), dM, xd, y)
            assert_parity(y.cpu().numpy(), y_ref, bound, f"COO,WM misaligned on {A.name}")


def test_coo_in_a_hip_graph_and_status_codes(cases):
    import torch
    A, x, y_ref, bound = next(c for c in cases if c[0].name.startswith("zipf1.6_20011"))
    dA, xd = upload(A), torch.from_numpy(x).cuda()
    plan = S.seer_spmv_prepare(S.COO_WM, dA)
    ws = S.alloc_workspace(S.spmv_prepared_workspace_bytes(plan))
    y = torch.full((A.rows,), float("nan"), device="cuda:0")
    S.seer_spmv_prepared(plan, dA, xd, y, ws)
    torch.cuda.synchronize()
    eager = y.clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        S.seer_spmv_prepared(plan, dA, xd, y, ws)
    for rep in range(3):
        y.fill_(float("nan"))
        _ = run_spmv(S.CSR_BM, dA, xd, A.rows)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, eager)
    assert_parity(y.cpu().numpy(), y_ref, bound, "COO,WM graph replay")
    with pytest.raises(S.SeerError) as ei:
        S.seer_spmv_prepare(S.COO_WM, dA, plan_mem=torch.empty(16, dtype=torch.uint8, device="cuda:0"))
    assert ei.value.status == -4
    with pytest.raises(S.SeerError) as ei:
        S.seer_spmv_prepared(plan, dA, xd, y, workspace=torch.empty(16, dtype=torch.uint8, device="cuda:0"))
    assert ei.value.status == -4
