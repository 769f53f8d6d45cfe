"""Two properties of the kernels as launched: (1) an Inf or NaN in x reaches exactly the rows
that hold its column -- the kernels fetch entries beyond a row's end (CSR,TM's eight-entry
window, the LDS-staged chunks, the padded ELL slots) and must never let such a foreign entry
into a row's sum; (2) calls on two streams with separate workspaces do not disturb each
other."""
import numpy as np
import pytest

import paper_2403_17017_amd as S
from workloads import csr_gen as G

from gpu_util import announce, assert_parity, oracle_of, upload

pytestmark = pytest.mark.gpu

# var_len <= 50 ? (mean_len <= 8 ? (rows <= 20000 ? TM : BM) : WM) : MP
TREE = ([6, 3, 0, -1, -1, -1, -1], [50.0, 8.0, 20000.0, 0, 0, 0, 0],
        [1, 2, 3, -1, -1, -1, -1], [6, 5, 4, -1, -1, -1, -1], [-1, -1, -1, 0, 2, 1, 3])


def poisoned_cases():
    out = []
    for A in (G.laplacian_5pt(150),                                # short rows: CSR,TM's window form, ELL width 5
              G.random_lengths(30_011, 20_000, 0, 12, 91),          # short rows, random columns, empty rows
              G.random_lengths(2_003, 9_000, 40, 300, 92),          # rows longer than a window, shorter than a chunk
              G.zipf_rows(25_000, s=1.5, cap=9_000, seed=93),       # rows across chunks and tiles: carries
              G.empty_poisson(60_000, 8_000, 0.3, 4.0, seed=94)):
        rng = np.random.default_rng(A.nnz)
        x = G.dense_vector(A.cols, 7)
        bad_cols = rng.choice(A.cols, size=3, replace=False)
        x_bad = x.copy()
        x_bad[bad_cols] = np.array([np.inf, np.nan, -np.inf], np.float32)
        hit = np.isin(A.col_idx[:A.nnz], bad_cols)
        row_of = np.repeat(np.arange(A.rows), np.diff(A.row_ptr.astype(np.int64)))
        touched = np.zeros(A.rows, bool)
        touched[row_of[hit]] = True
        assert 0 < touched.sum() < A.rows
        x_clean = x.copy()
        x_clean[bad_cols] = 0.0                 # what the untouched rows see either way
        y_ref, bound = oracle_of(A, x_clean)
        out.append((A, x_bad, touched, y_ref, bound))
    return out


@pytest.fixture(scope="module")
def poisoned():
    return poisoned_cases()


def check_poisoned(y, touched, y_ref, bound, what):
    clean = ~touched
    assert np.all(np.isfinite(y[clean])), f"{what}: {int((~np.isfinite(y[clean])).sum())} rows without a poisoned column are not finite"
    err = np.abs(y[clean].astype(np.float64) - y_ref[clean])
    assert np.all(err <= 1e-5 * bound[clean]), f"{what}: rows without a poisoned column are off by {err.max()}"
    assert not np.any(np.isfinite(y[touched])), f"{what}: a row that holds a poisoned column came out finite"


@pytest.mark.parametrize("kid", range(S.NUM_KERNELS))
def test_nonfinite_x_reaches_only_the_rows_that_hold_it(poisoned, kid, request):
    import torch
    if kid == S.CSR_S:                           # slabs of 1024 columns, so that these matrices are several slabs wide
        S.set_tuning("slab_shift", 10)
        request.addfinalizer(lambda: S.set_tuning("slab_shift", -1))
    for A, x_bad, touched, y_ref, bound in poisoned:
        announce(f"Inf/NaN in x, kernel {kid}, {A.name} rows={A.rows} nnz={A.nnz}")
        dA = upload(A)
        xd = torch.from_numpy(x_bad).cuda()
        y = torch.full((A.rows,), 12345.0, dtype=torch.float32, device="cuda:0")
        if kid in S.ONE_CALL_KERNELS:
            S.seer_spmv(kid, dA, xd, y)
            torch.cuda.synchronize()
            check_poisoned(y.cpu().numpy(), touched, y_ref, bound, f"seer_spmv kernel {kid} on {A.name}")
            y.fill_(12345.0)
        try:
            plan = S.seer_spmv_prepare(kid, dA)
        except S.SeerError:
            assert kid == S.ELL_TM               # padded form not applicable: nothing to run
            continue
        S.seer_spmv_prepared(plan, dA, xd, y)
        torch.cuda.synchronize()
        check_poisoned(y.cpu().numpy(), touched, y_ref, bound, f"prepared kernel {kid} on {A.name}")


def test_nonfinite_x_through_the_asynchronous_path(poisoned):
    import torch
    for A, x_bad, touched, y_ref, bound in poisoned:
        dA = upload(A)
        xd = torch.from_numpy(x_bad).cuda()
        ws = S.alloc_workspace(S.spmv_auto_workspace_bytes(A.rows, A.nnz))
        for tree in [S.Tree(*TREE)] + [S.Tree.constant(k) for k in range(S.NUM_DIRECT_KERNELS)]:
            for prune in (1, 0):                  # decided on the host / gathered and run by the combined kernel
                announce(f"Inf/NaN in x, seer_spmv_auto ({len(tree.arrays[0])}-node tree, prune={prune}), {A.name}")
                y = torch.full((A.rows,), 12345.0, dtype=torch.float32, device="cuda:0")
                S.set_tuning("auto_prune", prune)
                try:
                    S.seer_spmv_auto(dA, tree, xd, y, ws)
                finally:
                    S.set_tuning("auto_prune", -1)
                torch.cuda.synchronize()
                check_poisoned(y.cpu().numpy(), touched, y_ref, bound, f"seer_spmv_auto on {A.name}")


def test_two_streams_two_matrices_interleaved():
    """seer_spmv_auto calls on two streams, one matrix and one workspace per stream, issued
    alternately without waiting: every y of every round must be its own matrix's product."""
    import torch
    mats = [G.laplacian_5pt(700), G.zipf_rows(150_000, s=1.5, cap=40_000, seed=57)]
    tree = S.Tree(*TREE)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    side = []
    for A in mats:
        x = G.dense_vector(A.cols, 31)
        y_ref, bound = oracle_of(A, x)
        side.append((A, upload(A), torch.from_numpy(x).cuda(), y_ref, bound,
                     S.alloc_workspace(S.spmv_auto_workspace_bytes(A.rows, A.nnz))))
    rounds = 6
    ys = [[torch.full((A.rows,), float("nan"), dtype=torch.float32, device="cuda:0") for _ in range(rounds)]
          for A, *_ in side]
    torch.cuda.synchronize()
    announce("two streams, two matrices, interleaved seer_spmv_auto")
    for r in range(rounds):
        for s_i, (A, dA, xd, y_ref, bound, ws) in enumerate(side):
            S.seer_spmv_auto(dA, tree, xd, ys[s_i][r], ws, stream=streams[s_i])
    torch.cuda.synchronize()
    kids = []
    for s_i, (A, dA, xd, y_ref, bound, ws) in enumerate(side):
        _, kid = S.seer_spmv_auto_result(ws, stream=streams[s_i])
        kids.append(kid)
        first = ys[s_i][0].cpu().numpy()
        assert_parity(first, y_ref, bound, f"stream {s_i}, {A.name}")
        for r in range(1, rounds):
            assert torch.equal(ys[s_i][r], ys[s_i][0]), f"stream {s_i} round {r} differs from round 0 on {A.name}"
    assert kids == [S.CSR_BM, S.CSR_MP], kids     # the two streams ran different schedules
