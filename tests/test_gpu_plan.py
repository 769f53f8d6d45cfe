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
        assert S.spmv_prepared_workspace_bytes(plan) == (S.spmv_workspace_bytes(S.CSR_WO, A.rows, A.nnz) if split else 0)
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
