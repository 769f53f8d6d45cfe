"""GPU parity of seer_csr_check with the oracle's count of contract violations
(bit-exact: integer work).  The check only reads the two index arrays, so a matrix
with planted defects is safe to hand to it (and to nothing else)."""
import numpy as np
import pytest

import paper_2403_17017_amd as S
from oracle import seer_oracle as O
from workloads import csr_gen as G

from gpu_util import announce

pytestmark = pytest.mark.gpu


def device_counts(rows, cols, nnz, rp, ci):
    import torch
    d = S.DeviceCSR(rows, cols, torch.from_numpy(rp).cuda(),
                    torch.from_numpy(ci).cuda() if ci.size else torch.zeros(1, dtype=torch.int32, device="cuda:0"),
                    torch.zeros(max(nnz, 1), device="cuda:0"), nnz)
    return S.seer_csr_check(d)


def test_well_formed_matrices_pass():
    for A in (G.laplacian_5pt(300), G.fixed_degree(), G.random_lengths(200_001, 5000, 0, 40, seed=2),
              G.explicit_lengths([0, 0, 0, 100_000, 0, 1], 777, seed=4), G.explicit_lengths([0] * 5000, 10, seed=1)):
        announce(f"csr check, well formed: {A.name} rows={A.rows} nnz={A.nnz}")
        assert device_counts(A.rows, A.cols, A.nnz, A.row_ptr, A.col_idx) == (0, 0)


def test_small_defects_match_the_oracle():
    i32 = lambda *v: np.array(v, dtype=np.int32)
    ci = i32(0, 1, 2, 3)
    for rows, cols, nnz, rp, c in (
            (2, 4, 4, i32(1, 2, 4), ci), (2, 4, 4, i32(0, 2, 3), ci), (2, 4, 4, i32(0, 5, 4), ci),
            (3, 4, 4, i32(2, 1, 0, 3), ci), (2, 4, 4, i32(0, -1, 4), ci),
            (2, 4, 4, i32(0, 2, 4), i32(-1, 4, 2, 9)), (2, 0, 4, i32(0, 2, 4), ci), (0, 5, 0, i32(0), i32())):
        announce(f"csr check, small case rows={rows} rp={rp.tolist()} ci={c.tolist()}")
        want = O.csr_defects(rows, cols, nnz, rp, c)
        assert device_counts(rows, cols, nnz, rp, c) == want


def test_planted_defects_in_a_large_matrix_match_the_oracle():
    """Several grid-stride trips per lane, defects spread over many waves."""
    A = G.random_lengths(1_300_003, 40_000, 0, 9, seed=21)
    rng = np.random.default_rng(8)
    ci = A.col_idx.copy()
    where = rng.choice(A.nnz, 5000, replace=False)
    ci[where[:3000]] = A.cols + rng.integers(0, 2**20, 3000)
    ci[where[3000:]] = -1 - rng.integers(0, 2**20, 2000)
    rp = A.row_ptr.copy()
    hit = rng.choice(A.rows - 2, 700, replace=False) + 1
    rp[hit] = rp[hit + 1] + rng.integers(1, 50, 700).astype(np.int32)     # offsets pushed past their successors
    rp[0] = 3
    announce(f"csr check, planted defects rows={A.rows} nnz={A.nnz}")
    want = O.csr_defects(A.rows, A.cols, A.nnz, rp, ci)
    assert want[1] == 5000 and want[0] >= 700
    assert device_counts(A.rows, A.cols, A.nnz, rp, ci) == want
    # the same workspace again, now on the intact matrix: the counters start from zero
    import torch
    ws = S.alloc_workspace(16)
    vals = torch.zeros(A.nnz, device="cuda:0")
    d_bad = S.DeviceCSR(A.rows, A.cols, torch.from_numpy(rp).cuda(), torch.from_numpy(ci).cuda(), vals, A.nnz)
    d_ok = S.DeviceCSR(A.rows, A.cols, torch.from_numpy(A.row_ptr).cuda(), torch.from_numpy(A.col_idx).cuda(), vals, A.nnz)
    assert S.seer_csr_check(d_bad, ws) == want
    assert S.seer_csr_check(d_ok, ws) == (0, 0)


def test_status_codes():
    import torch
    A = G.laplacian_5pt(20)
    d = S.DeviceCSR.from_host(A)
    small = torch.zeros(8, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(S.SeerError) as ei:
        S.seer_csr_check(d, small)
    assert ei.value.status == -4
