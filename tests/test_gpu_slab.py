"""GPU parity of CSR,S, the column-slabbed schedule: the preprocessing's arrays against the
oracle's slab plan entry for entry, the product against the oracle's row sums, and the cases
in which the form does not apply."""
import numpy as np
import pytest

import paper_2403_17017_amd as S
from oracle import seer_oracle as O
from workloads import csr_gen as G

from gpu_util import announce, assert_parity, oracle_of, upload

pytestmark = pytest.mark.gpu


@pytest.fixture
def shift(request):
    S.set_tuning("slab_shift", request.param)
    yield request.param
    S.set_tuning("slab_shift", -1)


def small_cases():
    return [
        G.explicit_lengths([0, 7, 0, 0, 3, 0], 70, 4, "empties"),
        G.explicit_lengths([9] * 6, 40, 6, "few-columns-with-repeats"),
        G.explicit_lengths([0] * 500 + [30_000] + [0] * 500, 70_000, 7, "giant-row-among-empties"),
        G.explicit_lengths([33, 32, 31, 64, 65, 1, 0, 2048, 4097], 5_000, 13, "around-the-long-row-limit"),
        # rows beyond 4096 entries are copied segment by segment (1024 entries to a wave): whole and
        # ragged last segments, giant rows side by side, one at the very end of the matrix
        G.explicit_lengths([8192, 4097, 0, 5120, 7168, 3, 4096, 6000], 20_000, 31, "adjacent-giant-rows"),
        G.random_lengths(5_003, 3_000, 0, 40, 21),
        G.random_lengths(1_237, 9_000, 50, 700, 22),
        G.zipf_rows(20_011, s=1.6, cap=5_000, seed=23),
        G.laplacian_5pt(100),
        G.empty_poisson(100_003, 20_000, 0.3, 4.0, seed=25),
        G.banded(30_001, 9, 26),
    ]


def check_plan_and_product(A, sh):
    import torch
    want = O.slab_plan(A.rows, A.cols, A.row_ptr, A.col_idx, sh)
    dA = upload(A)
    if want is None:
        with pytest.raises(S.SeerError) as ei:
            S.seer_spmv_prepare(S.CSR_S, dA)
        assert ei.value.status == -1
        return False
    plan = S.seer_spmv_prepare(S.CSR_S, dA)
    assert plan.kernel_id == S.CSR_S and plan.n_blocks == want["n_slabs"]
    assert int(plan.c.split_rows) == len(want["rp_z"]) - 1, f"{A.name}: number of kept virtual rows"
    rp_z, p_idx, rp_j, ci, va = plan.slab_arrays(A.cols)
    assert np.array_equal(rp_z.astype(np.int64), want["rp_z"]), f"{A.name}: kept virtual rows' offsets differ"
    assert np.array_equal(rp_j.astype(np.int64), want["rp_j"]) and np.array_equal(p_idx.astype(np.int64), want["p_idx"]), \
        f"{A.name}: rows' piece lists differ"
    assert np.array_equal(ci, A.col_idx[want["perm"]]) and np.array_equal(va, A.values[want["perm"]]), \
        f"{A.name}: slabbed entries differ"
    x = G.dense_vector(A.cols, 3)
    y_ref, bound = oracle_of(A, x)
    y = torch.full((A.rows,), float("nan"), dtype=torch.float32, device="cuda:0")
    S.seer_spmv_prepared(plan, dA, torch.from_numpy(x).cuda(), y)
    torch.cuda.synchronize()
    assert_parity(y.cpu().numpy(), y_ref, bound, f"CSR,S on {A.name} (shift {sh})")
    return True


@pytest.mark.parametrize("shift", [3, 6, 10, 12], indirect=True)
def test_slab_plan_bit_exact_and_product_parity(shift):
    ran = 0
    for A in small_cases():
        announce(f"CSR,S shift={shift} {A.name} rows={A.rows} cols={A.cols} nnz={A.nnz}")
        ran += check_plan_and_product(A, shift)
    assert ran >= 5


def test_default_slab_size_on_a_matrix_with_several_slabs():
    """Slabs of 2^19 columns as shipped: 1.3 M columns are three slabs; rows of 0 to 30 entries."""
    A = G.random_lengths(300_007, 1_300_000, 0, 30, 77)
    announce(f"CSR,S default shift {A.name} rows={A.rows} cols={A.cols} nnz={A.nnz}")
    assert S.slab_plan_bytes(A.rows, A.cols, A.nnz) > 8 * A.nnz + 8 * 3 * A.rows
    assert check_plan_and_product(A, O.SLAB_SHIFT)


def test_random_matrices_and_slab_widths():
    """Eighty drawn matrices (short rows, mostly empty with rows of thousands, Zipf lengths, one
    giant row among near-empty ones) under drawn slab widths of 4 to 8192 columns: every plan
    entry for entry, every product against the oracle."""
    rng = np.random.default_rng(20261128)
    ran = 0
    try:
        for it in range(80):
            rows, cols = int(rng.integers(1, 6000)), int(rng.integers(2, 60000))
            kind = int(rng.integers(0, 4))
            if kind == 0:
                lens = rng.integers(0, min(cols, 40) + 1, rows)
            elif kind == 1:
                lens = np.where(rng.random(rows) < 0.7, 0, rng.integers(0, min(cols, 9000) + 1, rows))
            elif kind == 2:
                lens = np.minimum(rng.zipf(1.4, rows), min(cols, 20000))
            else:
                lens = rng.integers(0, 3, rows)
                lens[rng.integers(0, rows)] = min(cols, int(rng.integers(1000, 30000)))
            if lens.sum() > 2_000_000:
                lens = lens // 4
            A = G.explicit_lengths([int(v) for v in lens], cols, int(rng.integers(1 << 30)), f"drawn-{it}")
            sh = int(rng.integers(2, 14))
            S.set_tuning("slab_shift", sh)
            announce(f"CSR,S drawn case {it} kind={kind} shift={sh} rows={A.rows} cols={A.cols} nnz={A.nnz}")
            ran += check_plan_and_product(A, sh)
    finally:
        S.set_tuning("slab_shift", -1)
    assert ran >= 60


def test_wide_matrix_of_short_rows_takes_the_wider_slabs():
    """2.2 M columns are five slabs of 2^19; rows of 0 to 8 entries would fall into pieces of
    about one entry, so the library takes slabs of 2^20 columns (three of them), as the oracle's
    rule says, and the plan is the oracle's plan for that width."""
    A = G.random_lengths(2_200_003, 2_200_003, 0, 8, 78)
    sh = O.slab_shift_for(A.rows, A.cols, A.nnz)
    assert sh == O.SLAB_SHIFT + 1
    announce(f"CSR,S rule-chosen shift {sh} {A.name} rows={A.rows} cols={A.cols} nnz={A.nnz}")
    plan = S.seer_spmv_prepare(S.CSR_S, upload(A))
    assert int(plan.c.ell_width) == sh and plan.n_blocks == 3
    assert S.slab_plan_bytes(A.rows, A.cols, A.nnz) == int(plan.c.device_bytes)
    assert check_plan_and_product(A, sh)
    B = G.random_lengths(300_007, 2_200_003, 10, 30, 79)     # five slabs, 20 per row: stays at 2^19
    assert O.slab_shift_for(B.rows, B.cols, B.nnz) == O.SLAB_SHIFT
    plan = S.seer_spmv_prepare(S.CSR_S, upload(B))
    assert int(plan.c.ell_width) == O.SLAB_SHIFT and plan.n_blocks == 5


def test_where_the_slabbed_form_does_not_apply():
    import torch
    # one slab at the default size
    A = G.random_lengths(2_000, 3_000, 0, 9, 5)
    assert S.slab_plan_bytes(A.rows, A.cols, A.nnz) == 0
    with pytest.raises(S.SeerError) as ei:
        S.seer_spmv_prepare(S.CSR_S, upload(A))
    assert ei.value.status == -1
    # no one-call form
    with pytest.raises(S.SeerError) as ei:
        S.seer_spmv(S.CSR_S, upload(A), torch.zeros(A.cols, device="cuda:0"), torch.zeros(A.rows, device="cuda:0"))
    assert ei.value.status == -2
    S.set_tuning("slab_shift", 8)
    try:
        # a row whose columns descend: short (walked) and long (cut by searches)
        for n in (5, 200):
            B = G.random_lengths(300, 3_000, n, n, 6)
            ci = B.col_idx.copy()
            a = int(B.row_ptr[17])
            ci[a], ci[a + n - 1] = ci[a + n - 1], ci[a]
            if ci[a] == ci[a + n - 1]:
                continue
            bad = G.HostCSR(B.rows, B.cols, B.row_ptr, ci, B.values, f"descending-{n}")
            assert O.slab_plan(bad.rows, bad.cols, bad.row_ptr, bad.col_idx, 8) is None
            announce(f"CSR,S refuses {bad.name}")
            with pytest.raises(S.SeerError) as ei:
                S.seer_spmv_prepare(S.CSR_S, upload(bad))
            assert ei.value.status == -1
        # a column outside the matrix (the caller's contract, but the preprocessing writes by slab
        # number): refused, in a short row and in a long one
        for n in (5, 200):
            B = G.random_lengths(300, 3_000, n, n, 9)
            ci = B.col_idx.copy()
            ci[int(B.row_ptr[41]) + n - 1] = B.cols
            bad = G.HostCSR(B.rows, B.cols, B.row_ptr, ci, B.values, f"column-out-of-range-{n}")
            announce(f"CSR,S refuses {bad.name}")
            with pytest.raises(S.SeerError) as ei:
                S.seer_spmv_prepare(S.CSR_S, upload(bad))
            assert ei.value.status == -1
        # plan memory too small: the size needed comes back
        import ctypes as C
        dA = upload(A)
        cs = dA.c_struct()
        need = S.slab_plan_bytes(A.rows, A.cols, A.nnz)
        assert need > 0
        small = S.alloc_workspace(1024)
        c = S.binding.seer_plan()
        rc = S.lib().seer_spmv_prepare(S.CSR_S, C.byref(cs), small.data_ptr(), small.numel(), None, C.byref(c))
        assert rc == -4 and c.device_bytes == need and c.kernel_id == 0
    finally:
        S.set_tuning("slab_shift", -1)


def test_plan_falls_back_when_the_slabbed_form_is_chosen_but_cannot_be_built():
    """A model that always answers CSR,S: seer_spmv_plan prepares it where it applies and
    CSR,A where it does not (one slab; descending columns; no room)."""
    import torch
    model = S.Model(S.Tree.constant(S.CSR_S), S.Tree.constant(S.CSR_S), S.Tree([-1], [0.0], [-1], [-1], [0], n_classes=2))
    A = G.random_lengths(40_000, 2_000, 0, 20, 8)            # one slab at the default size
    dA = upload(A)
    plan, path = S.seer_spmv_plan(dA, model, 50)
    assert path == 0 and plan.kernel_id == S.CSR_A
    S.set_tuning("slab_shift", 7)
    try:
        plan, path = S.seer_spmv_plan(dA, model, 50)
        assert plan.kernel_id == S.CSR_S and plan.n_blocks == -(-2_000 // 128)
        x = G.dense_vector(A.cols, 4)
        y_ref, bound = oracle_of(A, x)
        y = torch.full((A.rows,), float("nan"), dtype=torch.float32, device="cuda:0")
        S.seer_spmv_prepared(plan, dA, torch.from_numpy(x).cuda(), y)
        torch.cuda.synchronize()
        assert_parity(y.cpu().numpy(), y_ref, bound, "planned CSR,S")
        tiny = S.alloc_workspace(S.plan_bytes(S.CSR_A, A.rows, A.nnz))   # room for CSR,A's plan only
        plan, path = S.seer_spmv_plan(dA, model, 50, plan_mem=tiny)
        assert plan.kernel_id == S.CSR_A
    finally:
        S.set_tuning("slab_shift", -1)
