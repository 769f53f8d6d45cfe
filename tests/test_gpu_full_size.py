"""GPU parity at the full sizes of the BASELINE configs, every row compared with the
oracle, in the launch configuration bench.py times (default launch shapes)."""
import numpy as np
import pytest

import paper_2403_17017_amd as S
from oracle import seer_oracle as O
from workloads import csr_gen as G

from gpu_util import announce, assert_features_equal, assert_parity, oracle_of, run_spmv, upload

pytestmark = pytest.mark.gpu


def check_all(A, kernels=(0, 1, 2, 3, 4, 5, 7), prepared=(5, 6, 7, 8)):
    import torch
    x = G.dense_vector(A.cols, 4242)
    y_ref, bound = oracle_of(A, x)
    dA = upload(A)
    xd = torch.from_numpy(x).cuda()
    announce(f"full size {A.name}: features")
    assert_features_equal(S.seer_features(dA), O.features(A.rows, A.cols, A.row_ptr), A.name)
    for kid in kernels:
        announce(f"full size {A.name}: kernel {kid} rows={A.rows} nnz={A.nnz}")
        y = run_spmv(kid, dA, xd, A.rows)
        assert_parity(y, y_ref, bound, f"kernel {kid} on {A.name}")
    for kid in prepared:
        announce(f"full size {A.name}: kernel {kid} from a prepared plan")
        plan = S.seer_spmv_prepare(kid, dA)
        y = torch.full((A.rows,), float("nan"), device="cuda:0")
        S.seer_spmv_prepared(plan, dA, xd, y)
        assert_parity(y.cpu().numpy(), y_ref, bound, f"prepared kernel {kid} on {A.name}")
        del plan
    return dA, xd


def test_config2_laplacian_1024():
    import torch
    A = G.laplacian_5pt(1024)
    dA, _ = check_all(A)
    # closed form on top of the oracle: x = 1 gives 4 - (number of neighbours), exactly
    ones = torch.ones(A.cols, device="cuda:0")
    r, c = np.divmod(np.arange(A.rows), 1024)
    want = (((r == 0) | (r == 1023)).astype(np.float32) + ((c == 0) | (c == 1023)).astype(np.float32))
    for kid in range(S.NUM_KERNELS):
        assert np.array_equal(run_spmv(kid, dA, ones, A.rows), want)


def test_config4_empty_rows_poisson_8M():
    A = G.empty_poisson()
    assert A.rows == 8_000_000 and A.cols == 1_000_000
    check_all(A)


def test_config3_zipf_nnz_matched():
    """Zipf exponent 1.85: the variant whose nonzero count (~47 M) matches the stated one."""
    A = G.zipf_rows(s=1.85)
    assert A.rows == 2_000_000 and int(np.diff(A.row_ptr).max()) == 200_000
    assert S.ell_plan_bytes(A.rows, 200_000) == 0          # ELL,TM does not apply to this matrix
    check_all(A, prepared=(5, 7, 8))


def test_config3_zipf_literal_parameters():
    """Zipf exponent 1.6 as stated (~4.8e8 nonzeros, 3.8 GB of entries)."""
    A = G.zipf_rows(s=1.6)
    assert A.nnz > 4e8 and int(np.diff(A.row_ptr).max()) == 200_000
    check_all(A, prepared=(5, 7, 8))


@pytest.mark.parametrize("workload", ["laplace5_1024", "empty30_poisson4_8M"])
def test_planned_products_at_full_size(workload):
    """seer_spmv_plan with the shipped models for 1, 19 and 100 products, then the product from
    the plan it returns, at the full size of BASELINE configs 2 and 4: the chosen kernel is what
    the oracle's three-tree inference says for that iteration count, y matches the oracle."""
    import os
    import torch
    from paper_2403_17017_amd import training as T
    A = G.laplacian_5pt(1024) if workload == "laplace5_1024" else G.empty_poisson()
    model_path = os.path.join(os.path.dirname(T.__file__), "selector_model.json")
    model, meta = T.load_model(model_path, iterative=True)
    x = G.dense_vector(A.cols, 99)
    y_ref, bound = oracle_of(A, x)
    dA = upload(A)
    xd = torch.from_numpy(x).cuda()
    for n in (1, 19, 100):
        announce(f"full size {A.name}: seer_spmv_plan for {n} products")
        plan, path = S.seer_spmv_plan(dA, model, n)
        fg = O.features(A.rows, A.cols, A.row_ptr, iterations=n)["f"]
        want_path, want_kid = O.model_select(A.rows, A.cols, A.nnz, fg, model.selector.arrays, model.known.arrays,
                                             model.gathered.arrays, iterations=n)
        assert path == want_path
        # (ELL,TM falls back to CSR,A where the plan memory cannot hold the padded form)
        assert plan.kernel_id == want_kid or (want_kid == S.ELL_TM and plan.kernel_id == S.CSR_A)
        y = torch.full((A.rows,), float("nan"), device="cuda:0")
        S.seer_spmv_prepared(plan, dA, xd, y)
        assert_parity(y.cpu().numpy(), y_ref, bound, f"{S.kernel_name(plan.kernel_id)} planned for {n} products on {A.name}")
        del plan


@pytest.mark.parametrize("extra", [1, 255, 256, 300, 511])
def test_thread_mapped_two_rows_per_lane_ragged_tail(extra):
    """From 2^20 short rows on CSR,TM takes two rows per lane (tiles of 512 rows): a last tile
    whose second half is partly or wholly beyond the matrix, stand-alone and inside the
    combined kernel of the asynchronous path."""
    import torch
    A = G.random_lengths((1 << 20) + extra, 70_001, 0, 6, seed=600 + extra)
    x = G.dense_vector(A.cols, 77)
    y_ref, bound = oracle_of(A, x)
    dA = upload(A)
    xd = torch.from_numpy(x).cuda()
    announce(f"two rows per lane, rows=2^20+{extra}: stand-alone")
    y = run_spmv(S.CSR_TM, dA, xd, A.rows)
    assert_parity(y, y_ref, bound, f"CSR,TM on 2^20+{extra} rows")
    announce(f"two rows per lane, rows=2^20+{extra}: combined kernel")
    ws = S.alloc_workspace(S.spmv_auto_workspace_bytes(A.rows, A.nnz))
    ya = torch.full((A.rows,), float("nan"), device="cuda:0")
    S.seer_spmv_auto(dA, S.Tree.constant(S.CSR_TM), xd, ya, ws)
    assert S.seer_spmv_auto_result(ws)[1] == S.CSR_TM
    assert np.array_equal(ya.cpu().numpy(), y)


def test_work_oriented_large_chunk_ragged():
    """From 2^23 nonzeros on CSR,WO takes chunks of 4096 nonzeros: a matrix just above that
    size with a ragged last chunk, empty rows, and rows that run through several chunks,
    stand-alone and inside the combined kernel."""
    import torch
    rng = np.random.default_rng(4096)
    lens = rng.integers(0, 57, 300_007)
    lens[rng.choice(lens.size, 40, replace=False)] = rng.integers(3_000, 30_000, 40)
    lens[1000:1400] = 0
    A = G.explicit_lengths(lens.tolist(), 90_001, seed=4097, name="just above 2^23 nonzeros")
    assert A.nnz >= (1 << 23) and A.nnz % 4096 != 0
    x = G.dense_vector(A.cols, 78)
    y_ref, bound = oracle_of(A, x)
    dA = upload(A)
    xd = torch.from_numpy(x).cuda()
    announce(f"large chunk, nnz={A.nnz}: stand-alone")
    y = run_spmv(S.CSR_WO, dA, xd, A.rows)
    assert_parity(y, y_ref, bound, "CSR,WO with 4096-nonzero chunks")
    announce(f"large chunk, nnz={A.nnz}: entry arrays 4 bytes off a 16-byte boundary (lane-strided loads)")
    y_mis = run_spmv(S.CSR_WO, upload(A, misalign=True), xd, A.rows)
    assert_parity(y_mis, y_ref, bound, "CSR,WO with 4096-nonzero chunks, misaligned entries")
    announce(f"large chunk, nnz={A.nnz}: combined kernel")
    ws = S.alloc_workspace(S.spmv_auto_workspace_bytes(A.rows, A.nnz))
    ya = torch.full((A.rows,), float("nan"), device="cuda:0")
    S.seer_spmv_auto(dA, S.Tree.constant(S.CSR_WO), xd, ya, ws)
    assert S.seer_spmv_auto_result(ws)[1] == S.CSR_WO
    assert np.array_equal(ya.cpu().numpy(), y)


@pytest.mark.timeout(1500)
def test_nnz_at_the_int32_limit():
    """The largest matrix the boundary accepts: nnz = 2^31 - 1 (the last value an int32
    offset can hold), 2 M rows of about a thousand entries, a tenth of them empty, one row
    of 5.5 M entries.  Every offset computation in the kernels must survive positions next
    to 2^31.  Values and x are small integers, so every row whose sum|a||x| stays below 2^24
    has to come out exactly, whatever order a schedule adds in; the one long row is held to
    the usual tolerance."""
    import torch
    announce("int32 limit: generating 16 GiB of entries on the host")
    A = G.int32_limit()
    assert A.nnz == 2**31 - 1
    x = np.random.default_rng(G.BASE_SEED + 32).integers(-4, 5, A.cols).astype(np.float32)
    announce("int32 limit: oracle")
    y_ref, bound = oracle_of(A, x)
    exact = bound < 2.0**24
    assert int(exact.sum()) >= A.rows - 1
    want = O.features(A.rows, A.cols, A.row_ptr)
    announce("int32 limit: upload")
    dA = upload(A)
    xd = torch.from_numpy(x).cuda()

    announce("int32 limit: input check and features")
    assert S.seer_csr_check(dA) == (0, 0)
    assert_features_equal(S.seer_features(dA), want, A.name)
    assert S.ell_plan_bytes(A.rows, int(want["max_len"])) == 0        # the padded form would not fit int32 either

    ys = {}
    for kid in (S.CSR_TM, S.CSR_WM, S.CSR_BM, S.CSR_MP, S.CSR_WO, S.CSR_A, S.COO_WM):
        announce(f"int32 limit: kernel {kid} ({S.kernel_name(kid)})")
        y = run_spmv(kid, dA, xd, A.rows)
        assert_parity(y, y_ref, bound, f"kernel {kid} at nnz = 2^31 - 1")
        assert np.array_equal(y[exact], y_ref[exact].astype(np.float32)), f"kernel {kid}: integer rows not exact"
        ys[kid] = y

    for kid in (S.CSR_MP, S.CSR_WO):
        announce(f"int32 limit: combined kernel answering {S.kernel_name(kid)}")
        ws = S.alloc_workspace(S.spmv_auto_workspace_bytes(A.rows, A.nnz))
        ya = torch.full((A.rows,), float("nan"), device="cuda:0")
        S.set_tuning("auto_prune", 0)          # gather although the one-leaf tree needs no features
        try:
            S.seer_spmv_auto(dA, S.Tree.constant(kid), xd, ya, ws)
        finally:
            S.set_tuning("auto_prune", -1)
        f_dev, kid_dev = S.seer_spmv_auto_result(ws)
        assert kid_dev == kid and f_dev.vector().tobytes() == want["f"].tobytes()
        assert np.array_equal(ya.cpu().numpy(), ys[kid])
        ya.fill_(float("nan"))                  # and decided on the host, nothing gathered
        S.seer_spmv_auto(dA, S.Tree.constant(kid), xd, ya, ws)
        f_dev, kid_dev = S.seer_spmv_auto_result(ws)
        assert kid_dev == kid and int(f_dev.max_len) == -1
        assert np.array_equal(ya.cpu().numpy(), ys[kid])
