"""seer_spmv_auto_static -- the entry point for callers that cannot allocate -- against
seer_spmv_auto, through the C ABI: two calls in a row on the library's one built-in scratch
array, the second with a smaller matrix, each bit-identical to the workspace form and within
tolerance of the oracle; then the size limit and a call with no rows."""
import pytest

import paper_2403_17017_amd as S
from workloads import csr_gen as G

from gpu_util import announce, assert_parity, oracle_of, upload

pytestmark = pytest.mark.gpu

# var_len <= 50 ? (mean_len <= 8 ? (rows <= 20000 ? TM : BM) : WM) : MP
TREE = ([6, 3, 0, -1, -1, -1, -1], [50.0, 8.0, 20000.0, 0, 0, 0, 0],
        [1, 2, 3, -1, -1, -1, -1], [6, 5, 4, -1, -1, -1, -1], [-1, -1, -1, 0, 2, 1, 3])


def both_forms(A, x, tree):
    import torch
    dA = upload(A)
    xd = torch.from_numpy(x).cuda()
    ws = S.alloc_workspace(S.spmv_auto_workspace_bytes(A.rows, A.nnz))
    y_ws = torch.full((A.rows,), float("nan"), dtype=torch.float32, device="cuda:0")
    y_st = torch.full((A.rows,), float("nan"), dtype=torch.float32, device="cuda:0")
    S.seer_spmv_auto(dA, tree, xd, y_ws, ws)
    _, kid = S.seer_spmv_auto_result(ws)
    S.seer_spmv_auto_static(dA, tree, xd, y_st)
    torch.cuda.synchronize()
    return y_ws.cpu().numpy(), y_st.cpu().numpy(), kid


def test_static_scratch_matches_workspace_form_twice():
    # a skewed matrix first (merge path: the carries fill the scratch far beyond what the second
    # call uses), then a small regular one (thread mapped) on the same, now dirty, array; then
    # the work-oriented schedule forced, whose fix-up reads carries again
    first = G.zipf_rows(120_000, s=1.5, cap=30_000, seed=41)
    second = G.laplacian_5pt(96)
    assert second.nnz < first.nnz and second.rows < first.rows
    for A, tree, want_kid in ((first, S.Tree(*TREE), S.CSR_MP), (second, S.Tree(*TREE), S.CSR_TM),
                              (second, S.Tree.constant(S.CSR_WO), S.CSR_WO)):
        announce(f"no-alloc entry point on {A.name} rows={A.rows} nnz={A.nnz}")
        x = G.dense_vector(A.cols, 77)
        y_ref, bound = oracle_of(A, x)
        y_ws, y_st, kid = both_forms(A, x, tree)
        assert kid == want_kid, f"{A.name}: the tree chose kernel {kid}"
        assert_parity(y_st, y_ref, bound, f"seer_spmv_auto_static on {A.name}")
        assert y_st.tobytes() == y_ws.tobytes(), f"static and workspace forms differ on {A.name}"


def test_static_scratch_limit_and_empty():
    import torch
    # beyond the built-in array: refused before anything is enqueued (the pointers are never used)
    rows, nnz = 1, 2_000_000_000
    assert S.spmv_auto_workspace_bytes(rows, nnz) > S.STATIC_SCRATCH_BYTES
    rp = torch.zeros(2, dtype=torch.int32, device="cuda:0")
    one = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    y = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    big = S.binding.seer_csr(rows, 1, nnz, rp.data_ptr(), rp.data_ptr(), one.data_ptr())
    rc = S.lib().seer_spmv_auto_static(big, S.Tree.constant(0).c, one.data_ptr(), y.data_ptr(), None)
    assert rc == -6 and "scratch" in S.strerror(rc)
    # no rows: accepted, nothing written
    none = S.binding.seer_csr(0, 5, 0, rp.data_ptr(), None, None)
    assert S.lib().seer_spmv_auto_static(none, S.Tree.constant(0).c, one.data_ptr(), y.data_ptr(), None) == 0
    torch.cuda.synchronize()
    assert float(y[0]) == 0.0
