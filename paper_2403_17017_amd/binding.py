"""ctypes binding of libseer.so: argument marshalling only.

Every step of the path -- feature reduction, tree walk, SpMV -- runs inside the
library; there is no Python or PyTorch fallback.  PyTorch supplies device memory
(``tensor.data_ptr()``) and the stream.  If the library has not been built the
first call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libseer.so")

NUM_FEATURES = 13
NUM_KERNELS = 9
NUM_DIRECT_KERNELS = 5          # ids below this need no preprocessing
CSR_TM, CSR_WM, CSR_BM, CSR_MP, CSR_WO, CSR_A, ELL_TM, COO_WM, CSR_S = range(9)
ONE_CALL_KERNELS = (CSR_TM, CSR_WM, CSR_BM, CSR_MP, CSR_WO, CSR_A, COO_WM)   # what seer_spmv accepts
FEATURE_NAMES = (
    "rows", "cols", "nnz", "mean_len", "max_len", "min_len", "var_len", "empty_frac",
    "mean_density", "max_density", "min_density", "var_density", "iterations",
)
F_ITERATIONS = 12


class SeerError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {status} ({strerror(status)})")
        self.status = status


class seer_csr(C.Structure):
    _fields_ = [("rows", C.c_int32), ("cols", C.c_int32), ("nnz", C.c_int32),
                ("row_ptr", C.c_void_p), ("col_idx", C.c_void_p), ("values", C.c_void_p)]


class seer_features_t(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("nnz", C.c_int64),
                ("max_len", C.c_int64), ("min_len", C.c_int64), ("empty_rows", C.c_int64),
                ("sum_sq_len", C.c_uint64), ("f", C.c_float * NUM_FEATURES)]

    def vector(self) -> np.ndarray:
        return np.array(list(self.f), dtype=np.float32)

    def as_dict(self) -> dict:
        d = {k: int(getattr(self, k)) for k in
             ("rows", "cols", "nnz", "max_len", "min_len", "empty_rows", "sum_sq_len")}
        d["f"] = self.vector()
        return d


class seer_node(C.Structure):
    _fields_ = [("feature", C.c_int32), ("left", C.c_int32), ("right", C.c_int32),
                ("klass", C.c_int32), ("threshold", C.c_double)]


class seer_model(C.Structure):
    pass


class seer_tree(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("n_features", C.c_int32), ("n_classes", C.c_int32),
                ("nodes", C.POINTER(seer_node))]


class seer_plan(C.Structure):
    _fields_ = [("kernel_id", C.c_int32), ("rows", C.c_int32), ("nnz", C.c_int32), ("n_blocks", C.c_int32),
                ("split_rows", C.c_int32), ("ell_width", C.c_int32), ("device", C.c_void_p),
                ("device_bytes", C.c_size_t)]


seer_model._fields_ = [("selector", C.POINTER(seer_tree)), ("known", C.POINTER(seer_tree)),
                       ("gathered", C.POINTER(seer_tree))]

_lib = None


def lib():
    """The loaded library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2403_17017_amd.build` "
                "(there is no non-HIP code path)")
        L = C.CDLL(LIB_PATH)
        vp, sz, i32 = C.c_void_p, C.c_size_t, C.c_int32
        L.seer_features.argtypes = [C.POINTER(seer_csr), C.POINTER(seer_features_t), vp, sz, vp]
        L.seer_features.restype = C.c_int
        L.seer_features_workspace_bytes.argtypes = [i32]
        L.seer_features_workspace_bytes.restype = sz
        L.seer_derive_features.argtypes = [C.POINTER(seer_features_t)]
        L.seer_derive_features.restype = C.c_int
        L.seer_known_features.argtypes = [i32, i32, i32, C.POINTER(seer_features_t)]
        L.seer_known_features.restype = C.c_int
        L.seer_select.argtypes = [C.POINTER(seer_features_t), C.POINTER(seer_tree), C.POINTER(C.c_int)]
        L.seer_select.restype = C.c_int
        L.seer_tree_reachable.argtypes = [C.POINTER(seer_tree), C.POINTER(seer_features_t), C.POINTER(C.c_uint32)]
        L.seer_tree_reachable.restype = C.c_int
        L.seer_spmv.argtypes = [C.c_int, C.POINTER(seer_csr), vp, vp, vp, sz, vp]
        L.seer_spmv.restype = C.c_int
        L.seer_spmv_workspace_bytes.argtypes = [C.c_int, i32, i32]
        L.seer_spmv_workspace_bytes.restype = sz
        L.seer_spmv_auto.argtypes = [C.POINTER(seer_csr), C.POINTER(seer_tree), vp, vp, vp, sz, vp]
        L.seer_spmv_auto.restype = C.c_int
        L.seer_spmv_auto_static.argtypes = [C.POINTER(seer_csr), C.POINTER(seer_tree), vp, vp, vp]
        L.seer_spmv_auto_static.restype = C.c_int
        L.seer_spmv_auto_workspace_bytes.argtypes = [i32, i32]
        L.seer_spmv_auto_workspace_bytes.restype = sz
        L.seer_spmv_auto_result.argtypes = [vp, vp, C.POINTER(seer_features_t), C.POINTER(C.c_int)]
        L.seer_spmv_auto_result.restype = C.c_int
        L.seer_spmv_model.argtypes = [C.POINTER(seer_csr), C.POINTER(seer_model), vp, vp, vp, sz, vp,
                                      C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.seer_spmv_model.restype = C.c_int
        L.seer_model_host_ns.argtypes = [C.POINTER(seer_model), i32, i32, i32, i32, C.POINTER(C.c_double)]
        L.seer_model_host_ns.restype = C.c_int
        L.seer_plan_bytes.argtypes = [C.c_int, i32, i32]
        L.seer_plan_bytes.restype = sz
        L.seer_ell_plan_bytes.argtypes = [i32, i32]
        L.seer_ell_plan_bytes.restype = sz
        L.seer_slab_plan_bytes.argtypes = [i32, i32, i32]
        L.seer_slab_plan_bytes.restype = sz
        L.seer_spmv_prepare.argtypes = [C.c_int, C.POINTER(seer_csr), vp, sz, vp, C.POINTER(seer_plan)]
        L.seer_spmv_prepare.restype = C.c_int
        L.seer_spmv_prepared.argtypes = [C.POINTER(seer_plan), C.POINTER(seer_csr), vp, vp, vp, sz, vp]
        L.seer_spmv_prepared.restype = C.c_int
        L.seer_spmv_prepared_workspace_bytes.argtypes = [C.POINTER(seer_plan)]
        L.seer_spmv_prepared_workspace_bytes.restype = sz
        L.seer_spmv_plan.argtypes = [C.POINTER(seer_csr), C.POINTER(seer_model), i32, vp, sz, vp, sz, vp,
                                     C.POINTER(seer_plan), C.POINTER(C.c_int)]
        L.seer_spmv_plan.restype = C.c_int
        L.seer_csr_check.argtypes = [C.POINTER(seer_csr), C.POINTER(C.c_int64), C.POINTER(C.c_int64), vp, sz, vp]
        L.seer_csr_check.restype = C.c_int
        L.seer_set_tuning.argtypes = [C.c_char_p, C.c_int]
        L.seer_set_tuning.restype = C.c_int
        L.seer_stream_copy.argtypes = [vp, vp, sz, vp]
        L.seer_stream_copy.restype = C.c_int
        L.seer_stream_sum.argtypes = [vp, sz, vp, vp]
        L.seer_stream_sum.restype = C.c_int
        L.seer_gather_sum.argtypes = [vp, vp, sz, vp, vp, vp]
        L.seer_gather_sum.restype = C.c_int
        L.seer_num_kernels.restype = C.c_int
        L.seer_kernel_name.argtypes = [C.c_int]
        L.seer_kernel_name.restype = C.c_char_p
        L.seer_strerror.argtypes = [C.c_int]
        L.seer_strerror.restype = C.c_char_p
        L.seer_last_hip_error.restype = C.c_int
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().seer_strerror(status).decode()


def kernel_name(kernel_id: int) -> str:
    s = lib().seer_kernel_name(kernel_id)
    return s.decode() if s else "?"


def set_tuning(name: str, value: int) -> None:
    rc = lib().seer_set_tuning(name.encode(), int(value))
    if rc:
        raise SeerError(rc, f"seer_set_tuning({name})")


@dataclass
class DeviceCSR:
    """CSR matrix whose three arrays are torch tensors on the GPU."""
    rows: int
    cols: int
    row_ptr: "torch.Tensor"   # int32 [rows + 1]
    col_idx: "torch.Tensor"   # int32 [nnz]
    values: "torch.Tensor"    # float32 [nnz]
    nnz: int = -1

    def __post_init__(self):
        import torch
        assert self.row_ptr.dtype == torch.int32 and self.col_idx.dtype == torch.int32
        assert self.values.dtype == torch.float32
        assert self.row_ptr.is_contiguous() and self.col_idx.is_contiguous() and self.values.is_contiguous()
        assert self.row_ptr.numel() == self.rows + 1
        if self.nnz < 0:
            self.nnz = int(self.col_idx.numel())
        assert self.col_idx.numel() >= self.nnz and self.values.numel() >= self.nnz

    @classmethod
    def from_host(cls, A, device="cuda:0") -> "DeviceCSR":
        import torch
        return cls(A.rows, A.cols,
                   torch.from_numpy(A.row_ptr).to(device),
                   torch.from_numpy(A.col_idx).to(device),
                   torch.from_numpy(A.values).to(device), A.nnz)

    def c_struct(self) -> seer_csr:
        return seer_csr(self.rows, self.cols, self.nnz, self.row_ptr.data_ptr(),
                        self.col_idx.data_ptr() if self.nnz else None,
                        self.values.data_ptr() if self.nnz else None)


class Tree:
    """Flat decision tree in host memory (node 0 = root, feature < 0 = leaf)."""

    def __init__(self, feature, threshold, left, right, klass, n_classes=NUM_KERNELS,
                 n_features=NUM_FEATURES):
        n = len(feature)
        self._nodes = (seer_node * n)()
        for i in range(n):
            self._nodes[i] = seer_node(int(feature[i]), int(left[i]), int(right[i]), int(klass[i]),
                                       float(threshold[i]))
        self.c = seer_tree(n, n_features, n_classes, C.cast(self._nodes, C.POINTER(seer_node)))
        self.arrays = (np.asarray(feature, np.int32), np.asarray(threshold, np.float64),
                       np.asarray(left, np.int32), np.asarray(right, np.int32), np.asarray(klass, np.int32))

    @classmethod
    def constant(cls, klass: int) -> "Tree":
        return cls([-1], [0.0], [-1], [-1], [klass])


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(int(stream.cuda_stream)) if hasattr(stream, "cuda_stream") else C.c_void_p(int(stream))


def features_workspace_bytes(rows: int) -> int:
    return int(lib().seer_features_workspace_bytes(rows))


def spmv_workspace_bytes(kernel_id: int, rows: int, nnz: int) -> int:
    return int(lib().seer_spmv_workspace_bytes(kernel_id, rows, nnz))


def alloc_workspace(nbytes: int, device="cuda:0"):
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _temporary_workspace(nbytes: int, device, stream):
    """Scratch for one asynchronous call, dropped by the caller as soon as the call has been
    enqueued: the allocator must not hand the block to other work before `stream` has run
    the kernels that use it.  On torch's current stream that is the allocator's own rule; a
    torch stream other than the current one is told with record_stream; a raw stream handle
    cannot be, so such a caller owns the workspace (as the C header asks of every caller)."""
    ws = alloc_workspace(nbytes, device)
    if stream is not None:
        if not hasattr(stream, "cuda_stream"):
            raise ValueError("pass workspace= when stream is a raw handle: a temporary one cannot be kept alive for it")
        ws.record_stream(stream)
    return ws


def seer_features(A: DeviceCSR, workspace=None, stream=None) -> seer_features_t:
    """Gathered features of A (runs the reduction kernel and waits for it)."""
    if workspace is None:
        workspace = alloc_workspace(features_workspace_bytes(A.rows), A.row_ptr.device)
    out = seer_features_t()
    cs = A.c_struct()
    rc = lib().seer_features(C.byref(cs), C.byref(out), workspace.data_ptr(), workspace.numel(),
                             _stream_ptr(stream))
    if rc:
        raise SeerError(rc, "seer_features")
    return out


def seer_csr_check(A: DeviceCSR, workspace=None, stream=None):
    """(bad offsets, bad column indices) of A, counted on the device; (0, 0) means every
    schedule may run on it.  Waits for the stream."""
    if workspace is None:
        workspace = alloc_workspace(16, A.row_ptr.device)
    bad_rp, bad_ci = C.c_int64(-1), C.c_int64(-1)
    cs = A.c_struct()
    rc = lib().seer_csr_check(C.byref(cs), C.byref(bad_rp), C.byref(bad_ci), workspace.data_ptr(),
                              workspace.numel(), _stream_ptr(stream))
    if rc:
        raise SeerError(rc, "seer_csr_check")
    return int(bad_rp.value), int(bad_ci.value)


def seer_derive_features(rows, cols, nnz, max_len, min_len, empty_rows, sum_sq_len) -> seer_features_t:
    io = seer_features_t(rows, cols, nnz, max_len, min_len, empty_rows, sum_sq_len)
    rc = lib().seer_derive_features(C.byref(io))
    if rc:
        raise SeerError(rc, "seer_derive_features")
    return io


def seer_known_features(rows: int, cols: int, nnz: int) -> seer_features_t:
    out = seer_features_t()
    rc = lib().seer_known_features(rows, cols, nnz, C.byref(out))
    if rc:
        raise SeerError(rc, "seer_known_features")
    return out


def seer_select(f: seer_features_t, tree: Tree) -> int:
    k = C.c_int(-1)
    rc = lib().seer_select(C.byref(f), C.byref(tree.c), C.byref(k))
    if rc:
        raise SeerError(rc, "seer_select")
    return int(k.value)


def seer_tree_reachable(tree: Tree, known: seer_features_t) -> set:
    """Classes the tree can still answer given the known features alone."""
    mask = C.c_uint32(0)
    rc = lib().seer_tree_reachable(C.byref(tree.c), C.byref(known), C.byref(mask))
    if rc:
        raise SeerError(rc, "seer_tree_reachable")
    return {k for k in range(32) if (mask.value >> k) & 1}


def seer_spmv(kernel_id: int, A: DeviceCSR, x, y, workspace=None, stream=None) -> None:
    """y = A x with schedule kernel_id; asynchronous on the stream."""
    import torch
    assert x.dtype == torch.float32 and y.dtype == torch.float32
    assert x.is_contiguous() and y.is_contiguous()
    assert x.numel() >= A.cols and y.numel() >= A.rows
    need = spmv_workspace_bytes(kernel_id, A.rows, A.nnz) if 0 <= kernel_id < NUM_KERNELS else 0
    if need and workspace is None:
        workspace = _temporary_workspace(need, A.row_ptr.device, stream)
    cs = A.c_struct()
    rc = lib().seer_spmv(int(kernel_id), C.byref(cs), x.data_ptr(), y.data_ptr(),
                         workspace.data_ptr() if workspace is not None else None,
                         workspace.numel() if workspace is not None else 0, _stream_ptr(stream))
    if rc:
        raise SeerError(rc, f"seer_spmv(kernel {kernel_id})")


def seer_stream_copy(dst, src, stream=None) -> None:
    """dst[:] = src with the library's plain copy kernel (measurement aid)."""
    assert dst.is_contiguous() and src.is_contiguous() and dst.element_size() == 4 == src.element_size()
    assert dst.numel() == src.numel()
    rc = lib().seer_stream_copy(dst.data_ptr(), src.data_ptr(), src.numel(), _stream_ptr(stream))
    if rc:
        raise SeerError(rc, "seer_stream_copy")


def seer_stream_sum(src, out64, stream=None) -> None:
    """Read-only pass over src with the library's checksum kernel (measurement aid)."""
    assert src.is_contiguous() and src.element_size() == 4 and out64.numel() * out64.element_size() >= 256
    rc = lib().seer_stream_sum(src.data_ptr(), src.numel(), out64.data_ptr(), _stream_ptr(stream))
    if rc:
        raise SeerError(rc, "seer_stream_sum")


def seer_gather_sum(idx, val, x, out64, stream=None) -> None:
    """sum val[k] * x[idx[k]] with streamed idx / val (measurement aid: the rate of gathers)."""
    assert idx.is_contiguous() and val.is_contiguous() and idx.numel() == val.numel()
    assert idx.element_size() == 4 == val.element_size() and out64.numel() * out64.element_size() >= 256
    rc = lib().seer_gather_sum(idx.data_ptr(), val.data_ptr(), idx.numel(), x.data_ptr(), out64.data_ptr(),
                               _stream_ptr(stream))
    if rc:
        raise SeerError(rc, "seer_gather_sum")


def spmv_auto_workspace_bytes(rows: int, nnz: int) -> int:
    return int(lib().seer_spmv_auto_workspace_bytes(rows, nnz))


def seer_spmv_auto(A: DeviceCSR, tree: Tree, x, y, workspace, stream=None) -> None:
    """Features, tree walk and SpMV enqueued back to back; returns without waiting."""
    cs = A.c_struct()
    rc = lib().seer_spmv_auto(C.byref(cs), C.byref(tree.c), x.data_ptr(), y.data_ptr(),
                              workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    if rc:
        raise SeerError(rc, "seer_spmv_auto")


STATIC_SCRATCH_BYTES = 2 << 20   # SEER_STATIC_SCRATCH_BYTES


def seer_spmv_auto_static(A: DeviceCSR, tree: Tree, x, y, stream=None) -> None:
    """seer_spmv_auto on the library's own built-in scratch: no workspace argument, nothing
    allocated.  Raises SeerError(SEER_ELIMIT) for a matrix beyond STATIC_SCRATCH_BYTES."""
    cs = A.c_struct()
    rc = lib().seer_spmv_auto_static(C.byref(cs), C.byref(tree.c), x.data_ptr(), y.data_ptr(), _stream_ptr(stream))
    if rc:
        raise SeerError(rc, "seer_spmv_auto_static")


def seer_spmv_auto_result(workspace, stream=None):
    """(features, kernel id) of the last seer_spmv_auto on this workspace (waits)."""
    f = seer_features_t()
    k = C.c_int(-1)
    rc = lib().seer_spmv_auto_result(workspace.data_ptr(), _stream_ptr(stream), C.byref(f), C.byref(k))
    if rc:
        raise SeerError(rc, "seer_spmv_auto_result")
    return f, int(k.value)


class Model:
    """The three trees of the classifier-selection scheme (selector may be None)."""

    def __init__(self, gathered: Tree, known: Tree = None, selector: Tree = None):
        self.gathered, self.known, self.selector = gathered, known, selector
        self.c = seer_model(C.pointer(selector.c) if selector is not None else None,
                            C.pointer(known.c) if known is not None else None,
                            C.pointer(gathered.c))


def seer_spmv_model(A: DeviceCSR, model: Model, x, y, workspace, stream=None):
    """Classifier-selection inference; returns (path, kernel_id): path 0 = known model
    (kernel_id valid), 1 = features gathered on the device (kernel_id -1)."""
    cs = A.c_struct()
    path, kid = C.c_int(-1), C.c_int(-1)
    rc = lib().seer_spmv_model(C.byref(cs), C.byref(model.c), x.data_ptr(), y.data_ptr(),
                               workspace.data_ptr(), workspace.numel(), _stream_ptr(stream),
                               C.byref(path), C.byref(kid))
    if rc:
        raise SeerError(rc, "seer_spmv_model")
    return int(path.value), int(kid.value)


def seer_model_host_ns(model: Model, rows: int, cols: int, nnz: int, reps: int = 2000) -> float:
    """Mean wall-clock nanoseconds of the host-side decision of seer_spmv_model (measurement aid)."""
    ns = C.c_double(0.0)
    rc = lib().seer_model_host_ns(C.byref(model.c), rows, cols, nnz, reps, C.byref(ns))
    if rc:
        raise SeerError(rc, "seer_model_host_ns")
    return float(ns.value)


class Plan:
    """A prepared kernel for one matrix: the host-side record plus the device memory
    the preprocessing wrote (kept alive here)."""

    def __init__(self, c: seer_plan, plan_mem):
        self.c, self.plan_mem = c, plan_mem

    kernel_id = property(lambda self: int(self.c.kernel_id))
    n_blocks = property(lambda self: int(self.c.n_blocks))
    ell_width = property(lambda self: int(self.c.ell_width))
    split_rows = property(lambda self: bool(self.c.split_rows))

    def ell_arrays(self):
        """(cols int32 [width, rows_pad], vals fp32 [width, rows_pad]) as host arrays."""
        import torch
        rows_pad = -(-int(self.c.rows) // 64) * 64
        n = rows_pad * self.ell_width
        half = int(self.c.device_bytes) // 2
        cols = self.plan_mem[: n * 4].view(torch.int32).cpu().numpy().reshape(self.ell_width, rows_pad)
        vals = self.plan_mem[half: half + n * 4].view(torch.float32).cpu().numpy().reshape(self.ell_width, rows_pad)
        return cols, vals

    def slab_arrays(self, cols: int):
        """(rp_z uint32 [K + 1], p_idx uint32 [K], rp_j uint32 [rows + 1], col_idx int32 [nnz],
        values fp32 [nnz]) of a CSR,S plan for a matrix of `cols` columns, as host arrays."""
        import torch
        rows, nnz, S_, K = int(self.c.rows), int(self.c.nnz), self.n_blocks, int(self.c.split_rows)
        pad = lambda b: (b + 255) & ~255
        m = min(nnz, S_ * rows)
        o_idx = pad((m + 1) * 4)
        o_j = o_idx + pad(m * 4 + 4)
        o_ci = o_j + pad((rows + 1) * 4)
        o_va = o_ci + pad(nnz * 4 + 4)
        u32 = lambda off, n: self.plan_mem[off: off + n * 4].view(torch.int32).cpu().numpy().view(np.uint32)
        ci = self.plan_mem[o_ci: o_ci + nnz * 4].view(torch.int32).cpu().numpy()
        va = self.plan_mem[o_va: o_va + nnz * 4].view(torch.float32).cpu().numpy()
        return u32(0, K + 1), u32(o_idx, K), u32(o_j, rows + 1), ci, va

    def coo_rows(self) -> np.ndarray:
        """Row index of every nonzero (int32 [nnz]) as a host array."""
        import torch
        return self.plan_mem[: int(self.c.nnz) * 4].view(torch.int32).cpu().numpy()

    def entries(self) -> np.ndarray:
        """The (first row, first nonzero) pairs as an int32 [n_blocks + 1, 2] host array."""
        import torch
        n = (self.n_blocks + 1) * 2
        return self.plan_mem[: n * 4].view(torch.int32).cpu().numpy().reshape(-1, 2)


def plan_bytes(kernel_id: int, rows: int, nnz: int) -> int:
    return int(lib().seer_plan_bytes(kernel_id, rows, nnz))


def ell_plan_bytes(rows: int, max_len: int) -> int:
    return int(lib().seer_ell_plan_bytes(rows, max_len))


def slab_plan_bytes(rows: int, cols: int, nnz: int) -> int:
    """Plan memory of CSR,S; 0 where the form does not apply by size."""
    return int(lib().seer_slab_plan_bytes(rows, cols, nnz))


def seer_spmv_prepare(kernel_id: int, A: DeviceCSR, plan_mem=None, stream=None, max_len: int = None) -> Plan:
    """Runs the preprocessing of kernel_id for A (waits for it) and returns the plan.
    For ELL_TM the plan memory is sized from max_len (the longest row) when none is given."""
    need = plan_bytes(kernel_id, A.rows, A.nnz)
    if kernel_id == ELL_TM and plan_mem is None:
        if max_len is None:
            max_len = int(seer_features(A, stream=stream).max_len)
        need = max(ell_plan_bytes(A.rows, max_len), features_workspace_bytes(A.rows))
    if kernel_id == CSR_S and plan_mem is None:
        need = slab_plan_bytes(A.rows, A.cols, A.nnz)
    if plan_mem is None and need:
        plan_mem = alloc_workspace(need, A.row_ptr.device)
    cs = A.c_struct()
    c = seer_plan()
    rc = lib().seer_spmv_prepare(int(kernel_id), C.byref(cs), plan_mem.data_ptr() if plan_mem is not None else None,
                                 plan_mem.numel() if plan_mem is not None else 0, _stream_ptr(stream), C.byref(c))
    if rc:
        raise SeerError(rc, f"seer_spmv_prepare(kernel {kernel_id})")
    return Plan(c, plan_mem)


def spmv_prepared_workspace_bytes(plan: Plan) -> int:
    return int(lib().seer_spmv_prepared_workspace_bytes(C.byref(plan.c)))


def seer_spmv_prepared(plan: Plan, A: DeviceCSR, x, y, workspace=None, stream=None) -> None:
    """y = A x with a prepared plan; asynchronous on the stream."""
    need = spmv_prepared_workspace_bytes(plan)
    if need and workspace is None:
        workspace = _temporary_workspace(need, A.row_ptr.device, stream)
    cs = A.c_struct()
    rc = lib().seer_spmv_prepared(C.byref(plan.c), C.byref(cs), x.data_ptr(), y.data_ptr(),
                                  workspace.data_ptr() if workspace is not None else None,
                                  workspace.numel() if workspace is not None else 0, _stream_ptr(stream))
    if rc:
        raise SeerError(rc, f"seer_spmv_prepared(kernel {plan.kernel_id})")


def seer_spmv_plan(A: DeviceCSR, model: Model, iterations: int, plan_mem=None, workspace=None, stream=None):
    """Selection for `iterations` products, then the chosen kernel's preprocessing.
    Returns (plan, path): path 0 = known model, 1 = features were gathered."""
    if plan_mem is None:
        # room for any kernel's plan: CSR,A's blocks, COO,WM's row indices (4 bytes per nonzero),
        # and the ELL arrays as long as padding adds at most half to the 8 bytes per nonzero
        # (beyond that the call prepares CSR,A instead, as the C header says)
        need = max(plan_bytes(CSR_A, A.rows, A.nnz), plan_bytes(COO_WM, A.rows, A.nnz), 12 * A.nnz + (1 << 20),
                   slab_plan_bytes(A.rows, A.cols, A.nnz))
        plan_mem = alloc_workspace(need, A.row_ptr.device)
    if workspace is None:
        workspace = alloc_workspace(features_workspace_bytes(A.rows), A.row_ptr.device)
    cs = A.c_struct()
    c = seer_plan()
    path = C.c_int(-1)
    rc = lib().seer_spmv_plan(C.byref(cs), C.byref(model.c), int(iterations), plan_mem.data_ptr(), plan_mem.numel(),
                              workspace.data_ptr(), workspace.numel(), _stream_ptr(stream), C.byref(c),
                              C.byref(path))
    if rc:
        raise SeerError(rc, "seer_spmv_plan")
    return Plan(c, plan_mem), int(path.value)
