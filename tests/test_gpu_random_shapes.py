"""GPU parity on many small random matrices of varied shape (seeded): every kernel of the
pool, one-call and from a prepared plan, against the oracle.  Shapes are drawn to hit what
the fixed cases may miss: row counts around the workgroup and wave sizes, nonzero counts
around the chunk sizes (512, 2048, 4096), leading / trailing / interleaved empty rows, a few
rows much longer than the rest."""
import numpy as np
import pytest

import paper_2403_17017_amd as S
from oracle import seer_oracle as O
from workloads import csr_gen as G

from gpu_util import announce, assert_features_equal, assert_parity, oracle_of, upload

pytestmark = pytest.mark.gpu



def prepare_or_none(kid, dA, A):
    """seer_spmv_prepare; for CSR,S with slabs small enough that the matrix has several (a
    sixteenth of the columns each), and None where the oracle says the form does not apply."""
    if kid != S.CSR_S:
        return S.seer_spmv_prepare(kid, dA)
    sh = max(1, int(A.cols).bit_length() - 4)
    S.set_tuning("slab_shift", sh)
    try:
        if O.slab_plan(A.rows, A.cols, A.row_ptr, A.col_idx, sh) is None:
            with pytest.raises(S.SeerError):
                S.seer_spmv_prepare(kid, dA)
            return None
        return S.seer_spmv_prepare(kid, dA)
    finally:
        S.set_tuning("slab_shift", -1)


def random_case(seed):
    rng = np.random.default_rng(9000 + seed)
    rows = int(rng.choice([1, 2, 63, 64, 65, 255, 256, 257, 1000, 4097, int(rng.integers(1, 6000))]))
    cols = int(rng.integers(1, 3000))
    kind = int(rng.integers(5))
    if kind == 0:      # short rows
        lens = rng.integers(0, 8, rows)
    elif kind == 1:    # mostly empty
        lens = (rng.random(rows) < 0.1) * rng.integers(1, 20, rows)
    elif kind == 2:    # a few long rows among short ones
        lens = rng.integers(0, 5, rows)
        for i in rng.integers(0, rows, 3):
            lens[i] = int(rng.choice([511, 512, 513, 2047, 2048, 2049, 4096, 4500, 9000]))
    elif kind == 3:    # nonzero count steered onto a chunk boundary
        lens = rng.integers(1, 6, rows)
        target = int(rng.choice([512, 2048, 4096, 6144])) * int(rng.integers(1, 3))
        lens[-1] += max(0, target - int(lens.sum()))
    else:              # wide rows
        lens = rng.integers(30, 200, rows)
    if rng.random() < 0.3:
        lens[: int(rng.integers(0, rows + 1))] = 0         # leading empty rows
    if rng.random() < 0.3:
        lens[rows - int(rng.integers(0, rows + 1)):] = 0   # trailing empty rows
    return G.explicit_lengths(np.asarray(lens, dtype=np.int64), cols, 9100 + seed, f"random#{seed}(kind {kind})")


@pytest.mark.parametrize("block", range(4))
def test_every_kernel_on_random_shapes(block):
    import torch
    for seed in range(block * 12, block * 12 + 12):
        A = random_case(seed)
        A.validate()
        x = G.dense_vector(A.cols, 9200 + seed)
        y_ref, bound = oracle_of(A, x)
        dA, xd = upload(A), torch.from_numpy(x).cuda()
        announce(f"{A.name} rows={A.rows} cols={A.cols} nnz={A.nnz} max_len={int(np.diff(A.row_ptr).max())}")
        assert_features_equal(S.seer_features(dA), O.features(A.rows, A.cols, A.row_ptr), A.name)
        for kid in range(S.NUM_KERNELS):
            if kid in S.ONE_CALL_KERNELS:
                y = torch.full((A.rows,), float("nan"), device="cuda:0")
                S.seer_spmv(kid, dA, xd, y)
                assert_parity(y.cpu().numpy(), y_ref, bound, f"{S.kernel_name(kid)} on {A.name}")
            plan = prepare_or_none(kid, dA, A)
            if plan is None:
                continue
            y = torch.full((A.rows,), float("nan"), device="cuda:0")
            S.seer_spmv_prepared(plan, dA, xd, y)
            assert_parity(y.cpu().numpy(), y_ref, bound, f"prepared {S.kernel_name(kid)} on {A.name}")
        # and the path that chooses for itself, with a tree that can reach every direct kernel
        tree = S.Tree([6, 3, 4, -1, -1, -1, 0, -1, -1], [1.0, 4.0, 600.0, 0, 0, 0, 300.0, 0, 0],
                      [1, 3, 5, -1, -1, -1, 7, -1, -1], [2, 4, 6, -1, -1, -1, 8, -1, -1],
                      [-1, -1, -1, 0, 1, 2, -1, 3, 4])
        ws = S.alloc_workspace(S.spmv_auto_workspace_bytes(A.rows, A.nnz))
        y = torch.full((A.rows,), float("nan"), device="cuda:0")
        S.seer_spmv_auto(dA, tree, xd, y, ws)
        f, kid = S.seer_spmv_auto_result(ws)
        assert kid == O.select(O.features(A.rows, A.cols, A.row_ptr)["f"], *tree.arrays)
        assert_parity(y.cpu().numpy(), y_ref, bound, f"seer_spmv_auto ({S.kernel_name(kid)}) on {A.name}")


def large_case(seed):
    """Sizes at which the launchers switch forms: two rows per lane and the round-robin tile
    order in CSR,TM (2^20 short rows; 96 MiB), 4096-nonzero chunks in CSR,WO (2^23 nonzeros),
    the guided first round of its row search (more than 4096 rows)."""
    rng = np.random.default_rng(9500 + seed)
    kind = seed % 4
    if kind == 0:      # short rows, a little over 2^20 of them, ragged last tile
        rows = (1 << 20) + int(rng.integers(1, 700))
        lens = rng.integers(0, 7, rows)
    elif kind == 1:    # short rows, large enough for the round-robin order
        rows = int(rng.integers(2_600_000, 3_000_000))
        lens = rng.integers(2, 9, rows)
    elif kind == 2:    # a little over 2^23 nonzeros, even rows
        rows = int(rng.integers(250_000, 300_000))
        lens = rng.integers(25, 40, rows)
        lens[-1] += max(0, (1 << 23) + int(rng.integers(1, 5000)) - int(lens.sum()))
    else:              # over 2^23 nonzeros, skewed, with runs of empty rows
        rows = int(rng.integers(400_000, 500_000))
        lens = np.minimum(rng.zipf(1.7, rows), 60_000)
        lens[rng.integers(0, rows, 200)] = rng.integers(2_000, 9_000, 200)
        lens[5000:9000] = 0
        lens[-1] += max(0, (1 << 23) + 17 - int(lens.sum()))
    cols = int(rng.integers(50_000, 400_000))
    return G.explicit_lengths(np.asarray(lens, dtype=np.int64), cols, 9600 + seed, f"large#{seed}(kind {kind})")


@pytest.mark.parametrize("seed", range(8))
def test_every_kernel_on_large_random_shapes(seed):
    import torch
    A = large_case(seed)
    x = G.dense_vector(A.cols, 9700 + seed)
    y_ref, bound = oracle_of(A, x)
    dA, xd = upload(A), torch.from_numpy(x).cuda()
    max_len = int(np.diff(A.row_ptr).max())
    announce(f"{A.name} rows={A.rows} cols={A.cols} nnz={A.nnz} max_len={max_len}")
    assert_features_equal(S.seer_features(dA), O.features(A.rows, A.cols, A.row_ptr), A.name)
    assert S.seer_csr_check(dA) == (0, 0)
    for kid in range(S.NUM_KERNELS):
        if kid in S.ONE_CALL_KERNELS:
            y = torch.full((A.rows,), float("nan"), device="cuda:0")
            S.seer_spmv(kid, dA, xd, y)
            assert_parity(y.cpu().numpy(), y_ref, bound, f"{S.kernel_name(kid)} on {A.name}")
        if kid == S.ELL_TM and not 0 < S.ell_plan_bytes(A.rows, max_len) <= (1 << 30):
            continue
        plan = prepare_or_none(kid, dA, A)
        if plan is None:
            continue
        y = torch.full((A.rows,), float("nan"), device="cuda:0")
        S.seer_spmv_prepared(plan, dA, xd, y)
        assert_parity(y.cpu().numpy(), y_ref, bound, f"prepared {S.kernel_name(kid)} on {A.name}")
        del plan
    ws = S.alloc_workspace(S.spmv_auto_workspace_bytes(A.rows, A.nnz))
    for forced in (S.CSR_TM if seed % 4 < 2 else S.CSR_WM, S.CSR_WO):
        y = torch.full((A.rows,), float("nan"), device="cuda:0")
        S.seer_spmv_auto(dA, S.Tree.constant(forced), xd, y, ws)
        assert S.seer_spmv_auto_result(ws)[1] == forced
        assert_parity(y.cpu().numpy(), y_ref, bound, f"seer_spmv_auto ({S.kernel_name(forced)}) on {A.name}")
