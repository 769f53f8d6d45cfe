"""Helpers shared by the GPU parity tests (not a test module)."""
import sys

import numpy as np

import paper_2403_17017_amd as S
from oracle import seer_oracle as O

TOL = 1e-5   # |y - y_ref| <= TOL * sum_k |a_ik| |x_k| per row (fp32 path against the fp64 oracle)


def announce(msg: str) -> None:
    """Name the case before GPU work starts, so a dead box still tells which one ran."""
    print(f"[gpu-case] {msg}", file=sys.stderr, flush=True)


def upload(A, misalign: bool = False):
    import torch
    if not misalign:
        return S.DeviceCSR.from_host(A)
    # entries start 4 bytes past a 16-byte boundary: forces the scalar-load kernels
    ci = torch.empty(A.nnz + 1, dtype=torch.int32, device="cuda:0")
    va = torch.empty(A.nnz + 1, dtype=torch.float32, device="cuda:0")
    ci[1:] = torch.from_numpy(A.col_idx).cuda()
    va[1:] = torch.from_numpy(A.values).cuda()
    d = S.DeviceCSR(A.rows, A.cols, torch.from_numpy(A.row_ptr).cuda(), ci[1:], va[1:], A.nnz)
    assert d.col_idx.data_ptr() % 16 == 4
    return d


def run_spmv(kernel_id, dA, x_dev, rows, poison=True):
    import torch
    y = torch.full((max(rows, 1),), float("nan"), dtype=torch.float32, device="cuda:0") if poison \
        else torch.zeros(max(rows, 1), dtype=torch.float32, device="cuda:0")
    if kernel_id in S.ONE_CALL_KERNELS:
        S.seer_spmv(kernel_id, dA, x_dev, y)
    else:                                      # preprocessing first (ELL,TM has no one-call form)
        S.seer_spmv_prepared(S.seer_spmv_prepare(kernel_id, dA), dA, x_dev, y)
    torch.cuda.synchronize()
    return y[:rows].cpu().numpy()


def assert_parity(y, y_ref, bound, what):
    assert y.shape == y_ref.shape, what
    assert not np.any(np.isnan(y)), f"{what}: {int(np.isnan(y).sum())} rows never written (or NaN)"
    err = np.abs(y.astype(np.float64) - y_ref)
    bad = err > TOL * bound
    if np.any(bad):
        i = int(np.argmax(err - TOL * bound))
        raise AssertionError(f"{what}: {int(bad.sum())} rows off; worst row {i}: got {y[i]!r} want {y_ref[i]!r} "
                             f"err {err[i]:.3e} allowed {TOL * bound[i]:.3e}")


def oracle_of(A, x):
    return O.spmv(A.rows, A.row_ptr, A.col_idx, A.values, x)


def assert_features_equal(got, want, what):
    for k in ("rows", "cols", "nnz", "max_len", "min_len", "empty_rows", "sum_sq_len"):
        assert int(getattr(got, k)) == int(want[k]), f"{what}: {k} {getattr(got, k)} != {want[k]}"
    assert got.vector().tobytes() == want["f"].tobytes(), f"{what}: f[] {got.vector()} != {want['f']}"
