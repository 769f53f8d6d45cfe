"""CPU oracle for the Seer SpMV hot path.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
module; the product library never does, and this module never imports the
product.  It is deliberately plain and slow.

What it defines
  * spmv        -- y = A x by the inner-product definition (Sec. IV, Table II:
                   every schedule computes the same SpMV), fp64, via the C row
                   loop in spmv_oracle.c; spmv_python is the same loop in Python
                   for tiny inputs.  spmv_all_cores is the same row loop with the rows
                   shared among the host threads (spmv_oracle_omp.c): a timed baseline
                   only, pinned bit for bit to the single-thread loop.
  * features    -- the statistics gathered from the CSR offsets (Sec. IV and
                   IV-A: max / min / variance / mean of the row density, where a
                   row's density is its nonzero count over the number of columns;
                   Table III's rows, nnz, Most, Least, Avg, Var), plus the
                   row-length forms of the same statistics and the fraction of
                   empty rows.
  * select      -- decision-tree inference (Sec. III-B: nested if/else over the
                   feature vector, returning an integer class index).
  * known_features, model_select -- the feature vector that costs nothing
                   (Sec. III-A) and inference with the classifier-selection
                   model that chooses between the known and the gathered model
                   (Sec. III-B).  The number of SpMV iterations the caller is
                   about to run is one more known feature (Sec. IV-E, multiple
                   iteration evaluation); it is 1 unless stated.
  * reachable_classes -- which kernels the gathered model can still answer once the
                   known features are fixed: what decides, before anything is gathered,
                   whether gathering can change the choice at all (Sec. III-B).
  * ell_from_csr -- the preprocessing result of the ELL,TM kernel (Table II: thread
                   mapped over "one row or fixed width" in the ELL format): every row
                   padded to the longest row's length, stored column-major.  The
                   layout (padding marker, row padding) is this build's; ell_spmv_python
                   multiplies from it literally.
  * coo_rows_from_csr -- the preprocessing result of the COO,WM kernel (Table II: warp
                   mapped over the COO format): the row index of every nonzero, in CSR
                   order.  coo_spmv_python multiplies from (row, col, value) triples.
  * adaptive_plan -- the preprocessing result of the Adaptive-CSR schedule
                   (Sec. IV: rows are grouped by size ahead of the first
                   product): row blocks of about `chunk` nonzeros, long rows
                   split between blocks.  The paper gives no data structure;
                   the one defined here is this build's reading, and
                   plan_spmv_python executes it literally so that tests can
                   check it assigns every nonzero to its row exactly once.

  * slab_plan -- the preprocessing result of the column-slabbed schedule: every row cut
                   into one virtual row per slab of 2^19 columns, entries stored slab after
                   slab, so that the gathers of one stretch of the matrix stay inside one
                   slab of x.  slab_spmv_python multiplies from it literally.

  * csr_defects -- the input contract of the kernels (Sec. IV-A: they consume the CSR
                   offsets and entries as given), counted: how many offsets and how
                   many column indices break it.  Not part of the paper's method; the
                   definition is the contract itself, written out.

Readings where the paper is silent (all listed again in the design document):
  * variance is the population variance (divide by rows);
  * integer statistics are exact; every derived float is computed in fp64 from
    exact integers with one division, then rounded once to fp32:
        mean_len   = fl32( fl64(nnz) / fl64(rows) )
        var_len    = fl32( fl64(rows*sum_sq - nnz^2) / fl64(rows^2) )
        empty_frac = fl32( fl64(empty) / fl64(rows) )
        densities  = the same fp64 quotient divided once more by fl64(cols)
                     (variance: by fl64(cols)*fl64(cols)), then rounded to fp32
    with fl64(int) the correctly rounded int->double conversion;
  * min is the plain minimum (0 if any row is empty);
  * rows == 0: every statistic and derived value is 0; cols == 0: densities 0;
  * tree split convention is scikit-learn's: go left iff x[feature] <= threshold,
    features fp32, thresholds fp64, comparison in fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

NUM_FEATURES = 13
FEATURE_NAMES = (
    "rows", "cols", "nnz", "mean_len", "max_len", "min_len", "var_len", "empty_frac",
    "mean_density", "max_density", "min_density", "var_density", "iterations",
)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile spmv_oracle.c with gcc (-O2, no OpenMP, no fast-math)."""
    src = os.path.join(_HERE, "spmv_oracle.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-o", _SO, src, "-lm"])
    return _SO


_SO_OMP = os.path.join(_HERE, "liboracle_omp.so")
_lib_omp = None


def build_all_cores(force: bool = False) -> str:
    """Compile spmv_oracle_omp.c (the same row loop, rows shared among the host threads)."""
    src = os.path.join(_HERE, "spmv_oracle_omp.c")
    if force or not os.path.exists(_SO_OMP) or os.path.getmtime(_SO_OMP) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _SO_OMP, src])
    return _SO_OMP


def spmv_all_cores(rows, row_ptr, col_idx, values, x):
    """The row loop of O1 on all host threads: a timed baseline, never the value checked
    against.  Returns (y fp64 [rows], threads used)."""
    global _lib_omp
    _check_csr(rows, row_ptr, col_idx, values, x)
    if _lib_omp is None:
        build_all_cores()
        lib = ctypes.CDLL(_SO_OMP)
        p = ctypes.c_void_p
        lib.oracle_spmv_f64_all_cores.argtypes = [ctypes.c_int64, p, p, p, p, p]
        lib.oracle_spmv_f64_all_cores.restype = ctypes.c_int
        _lib_omp = lib
    y = np.empty(rows, dtype=np.float64)
    ptr = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    threads = _lib_omp.oracle_spmv_f64_all_cores(rows, ptr(row_ptr), ptr(col_idx), ptr(values), ptr(x), ptr(y))
    return y, int(threads)


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_SO)
        p = ctypes.c_void_p
        lib.oracle_spmv_f64.argtypes = [ctypes.c_int64, p, p, p, p, p, p]
        lib.oracle_spmv_f64.restype = None
        lib.oracle_spmv_f64_nobound.argtypes = [ctypes.c_int64, p, p, p, p, p]
        lib.oracle_spmv_f64_nobound.restype = None
        _lib = lib
    return _lib


def _check_csr(rows, row_ptr, col_idx, values, x):
    assert row_ptr.dtype == np.int32 and row_ptr.flags.c_contiguous and row_ptr.shape == (rows + 1,)
    nnz = int(row_ptr[rows]) if rows >= 0 else 0
    assert col_idx.dtype == np.int32 and col_idx.flags.c_contiguous and col_idx.size >= nnz
    assert values.dtype == np.float32 and values.flags.c_contiguous and values.size >= nnz
    assert x.dtype == np.float32 and x.flags.c_contiguous
    if nnz:
        assert int(col_idx[:nnz].min()) >= 0 and int(col_idx[:nnz].max()) < x.size


def spmv(rows, row_ptr, col_idx, values, x, want_bound: bool = True):
    """O1.  Returns (y_ref fp64 [rows], bound fp64 [rows] or None)."""
    _check_csr(rows, row_ptr, col_idx, values, x)
    y = np.empty(rows, dtype=np.float64)
    lib = _load()
    ptr = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    if want_bound:
        b = np.empty(rows, dtype=np.float64)
        lib.oracle_spmv_f64(rows, ptr(row_ptr), ptr(col_idx), ptr(values), ptr(x), ptr(y), ptr(b))
        return y, b
    lib.oracle_spmv_f64_nobound(rows, ptr(row_ptr), ptr(col_idx), ptr(values), ptr(x), ptr(y))
    return y, None


def spmv_python(rows, row_ptr, col_idx, values, x):
    """O1 again as a pure-Python loop (Python floats are fp64); tiny inputs only."""
    y = [0.0] * rows
    bound = [0.0] * rows
    for i in range(rows):
        s = 0.0
        b = 0.0
        for k in range(int(row_ptr[i]), int(row_ptr[i + 1])):
            p = float(values[k]) * float(x[int(col_idx[k])])
            s += p
            b += abs(p)
        y[i] = s
        bound[i] = b
    return np.array(y, dtype=np.float64), np.array(bound, dtype=np.float64)


def _f32(v: float) -> np.float32:
    return np.float32(np.float64(v))


def features(rows: int, cols: int, row_ptr, iterations: int = 1) -> dict:
    """O2.  One pass over the CSR offsets; exact integers, then the derived vector."""
    out = dict(rows=int(rows), cols=int(cols), nnz=0, max_len=0, min_len=0,
               empty_rows=0, sum_sq_len=0)
    f = np.zeros(NUM_FEATURES, dtype=np.float32)
    if rows > 0:
        rp = np.asarray(row_ptr[: rows + 1], dtype=np.int64)
        lens = rp[1:] - rp[:-1]
        nnz = int(rp[rows] - rp[0])
        max_len = int(lens.max())
        min_len = int(lens.min())
        empty = int(np.count_nonzero(lens == 0))
        # len < 2^31 and sum(len) < 2^31, so sum(len^2) <= max*nnz < 2^62: exact in uint64
        sum_sq = int(np.sum(lens.astype(np.uint64) ** 2, dtype=np.uint64))
        out.update(nnz=nnz, max_len=max_len, min_len=min_len, empty_rows=empty, sum_sq_len=sum_sq)

        R = float(rows)                       # exact for rows < 2^53
        mean64 = float(nnz) / R
        var_num = rows * sum_sq - nnz * nnz   # Python int: exact, >= 0 (Cauchy-Schwarz)
        var64 = float(var_num) / float(rows * rows)
        f[0] = _f32(float(rows)); f[1] = _f32(float(cols)); f[2] = _f32(float(nnz))
        f[3] = _f32(mean64)
        f[4] = _f32(float(max_len))
        f[5] = _f32(float(min_len))
        f[6] = _f32(var64)
        f[7] = _f32(float(empty) / R)
        if cols > 0:
            C = float(cols)
            f[8] = _f32(mean64 / C)
            f[9] = _f32(float(max_len) / C)
            f[10] = _f32(float(min_len) / C)
            f[11] = _f32(var64 / (C * C))
    else:
        f[1] = _f32(float(cols))
    f[12] = _f32(float(iterations))
    out["f"] = f
    return out


def known_features(rows: int, cols: int, nnz: int, iterations: int = 1) -> np.ndarray:
    """The feature vector of a known-features model (Sec. III-A: rows, columns and
    nonzeros come with the dataset at no cost).  The mean row length and mean row
    density follow from those three numbers alone, so they are known as well; every
    entry that needs a look at the matrix stays 0."""
    f = np.zeros(NUM_FEATURES, dtype=np.float32)
    f[0] = _f32(float(rows)); f[1] = _f32(float(cols)); f[2] = _f32(float(nnz))
    if rows > 0:
        mean64 = float(nnz) / float(rows)
        f[3] = _f32(mean64)
        if cols > 0:
            f[8] = _f32(mean64 / float(cols))
    f[12] = _f32(float(iterations))
    return f


def model_select(rows, cols, nnz, f_gathered, selector, known, gathered, iterations: int = 1):
    """Classifier-selection inference (Sec. III-B).  Each tree is a 5-tuple of parallel
    arrays; selector may be None (always gather).  Returns (path, kernel id) with
    path 0 = known model, 1 = gathered model.  f_gathered must carry the same
    iteration count in its last entry."""
    if selector is not None:
        kf = known_features(rows, cols, nnz, iterations)
        if select(kf, *selector) == 0:
            return 0, select(kf, *known)
    return 1, select(f_gathered, *gathered)


KNOWN_FEATURES = (0, 1, 2, 3, 8, 12)   # rows, cols, nnz, mean_len, mean_density, iterations


def reachable_classes(f_known, feature, threshold, left, right, klass) -> set:
    """The classes a walk of the tree (as in select) can end in when only the known
    entries of the feature vector are fixed (Sec. III-A: the features that come with the
    dataset at no cost) and every gathered entry may take any value: at a node that tests a
    known entry the walk goes where select would go; at a node that tests a gathered entry
    both children stay possible.  Comparisons on the same gathered entry along one path are
    not reconciled with each other, so the set can hold a class no real vector reaches; it
    never misses one.  A single class means the matrix need not be looked at (Sec. III-B:
    feature collection is paid for only where it is justified)."""
    out = set()

    def walk(n):
        if int(feature[n]) < 0:
            out.add(int(klass[n]))
        elif int(feature[n]) in KNOWN_FEATURES:
            walk(int(left[n]) if float(np.float32(f_known[int(feature[n])])) <= float(threshold[n]) else int(right[n]))
        else:
            walk(int(left[n]))
            walk(int(right[n]))

    walk(0)
    return out


def select(f, feature, threshold, left, right, klass) -> int:
    """O3.  Walk a binary decision tree stored as parallel arrays; node 0 is the
    root; a node with feature < 0 is a leaf and returns klass[node]."""
    n = 0
    steps = 0
    while int(feature[n]) >= 0:
        n = int(left[n]) if float(np.float32(f[int(feature[n])])) <= float(threshold[n]) else int(right[n])
        steps += 1
        if steps > len(feature):
            raise ValueError("tree has a cycle")
    return int(klass[n])


def adaptive_plan(rows: int, row_ptr, chunk: int):
    """Row blocks of the Adaptive-CSR schedule.  With n = max(1, ceil(nnz / chunk))
    blocks, block k covers rows [row[k], row[k+1]) and nonzeros [start[k], start[k+1]):
        row[0] = 0, start[0] = 0, row[n] = rows, start[n] = nnz, and for 0 < k < n
        row[k]   = the first row that ends after nonzero k*chunk,
        start[k] = k*chunk      if that row is also row[k-1] (the row runs through the
                                whole of block k-1, which then holds nothing else),
                   row_ptr[row[k]] otherwise (blocks begin on a row boundary).
    A block with row[k] == row[k+1] lies inside one long row and contributes a partial
    sum to it; every other row is summed by the one block that holds its end.
    Returns (row, start) as int64 arrays of n + 1 entries; rows == 0 gives n = 0."""
    if rows == 0:
        return np.zeros(1, np.int64), np.zeros(1, np.int64)
    rp = np.asarray(row_ptr[: rows + 1], dtype=np.int64)
    nnz = int(rp[rows])
    n = max(1, -(-nnz // chunk))
    row = np.zeros(n + 1, np.int64)
    start = np.zeros(n + 1, np.int64)
    ends = rp[1:].tolist()
    i = 0
    for k in range(1, n):
        while ends[i] <= k * chunk:             # rows that end at or before nonzero k*chunk
            i += 1                              # (row ends never decrease, so i only moves forward)
        row[k] = i
        start[k] = k * chunk if row[k - 1] == i else int(rp[i])
    row[n] = rows
    start[n] = nnz
    return row, start


def plan_spmv_python(rows, row_ptr, col_idx, values, x, row, start):
    """Executes a plan literally, block by block, in exact Python arithmetic on whatever
    number type the inputs hold (tests use small integers): the rows a block owns take
    the part of themselves that lies inside the block's nonzero range, a block inside
    one long row adds its whole range to that row."""
    y = [0] * rows
    for k in range(len(row) - 1):
        lo, hi, s, e = int(row[k]), int(row[k + 1]), int(start[k]), int(start[k + 1])
        if lo == hi:
            y[lo] += sum(values[j] * x[col_idx[j]] for j in range(s, e))
            continue
        for i in range(lo, hi):
            a, b = max(int(row_ptr[i]), s), min(int(row_ptr[i + 1]), e)
            y[i] += sum(values[j] * x[col_idx[j]] for j in range(a, b))
    return y


ELL_ROW_MULTIPLE = 64      # rows are padded to a multiple of this (one wave of lanes)


def ell_from_csr(rows: int, row_ptr, col_idx, values):
    """ELL form of a CSR matrix: width = the longest row; cols[j, i] / vals[j, i] hold the
    j-th entry of row i in CSR order, cols = -1 and vals = 0 where row i has fewer than
    j + 1 entries; the row dimension is padded to a multiple of ELL_ROW_MULTIPLE (padding
    rows are all -1 / 0).  Returns (cols int32 [width, rows_pad], vals fp32 [width, rows_pad])."""
    rp = np.asarray(row_ptr[: rows + 1], dtype=np.int64)
    width = int((rp[1:] - rp[:-1]).max()) if rows > 0 else 0
    rows_pad = -(-rows // ELL_ROW_MULTIPLE) * ELL_ROW_MULTIPLE
    cols = np.full((width, rows_pad), -1, dtype=np.int32)
    vals = np.zeros((width, rows_pad), dtype=np.float32)
    for i in range(rows):
        a, b = int(rp[i]), int(rp[i + 1])
        cols[: b - a, i] = col_idx[a:b]
        vals[: b - a, i] = values[a:b]
    return cols, vals


def ell_spmv_python(rows, cols, vals, x):
    """y = A x from the ELL arrays, entry by entry, padding skipped (not multiplied: a
    padded slot must not turn an infinite x into NaN)."""
    y = [0] * rows
    for i in range(rows):
        for j in range(cols.shape[0]):
            c = int(cols[j, i])
            if c >= 0:
                y[i] += vals[j, i].item() * x[c]
    return y


def coo_rows_from_csr(rows: int, row_ptr) -> np.ndarray:
    """Row index of every nonzero, in CSR order (int32 [nnz]): the third array of the COO
    form; columns and values are the CSR arrays themselves."""
    rp = np.asarray(row_ptr[: rows + 1], dtype=np.int64)
    out = np.zeros(int(rp[rows]) if rows > 0 else 0, dtype=np.int32)
    for i in range(rows):
        out[int(rp[i]): int(rp[i + 1])] = i
    return out


def coo_spmv_python(rows, coo_row, col_idx, values, x):
    """y = A x from the triples: y starts at zero (a row without a triple stays zero) and
    every triple adds its product to its row."""
    y = [0] * rows
    for r, c, v in zip(coo_row, col_idx, values):
        y[int(r)] += v * x[int(c)]
    return y


SLAB_SHIFT = 19      # a slab of x holds 2^19 columns = 2 MiB, half of one XCD's L2


def slab_shift_for(rows: int, cols: int, nnz: int) -> int:
    """Which slab width the column-slabbed schedule takes for a matrix of this shape (a
    choice of this build, like the format itself): 2^19 columns, but 2^20 where that width would
    give at least four slabs and the rows are so short that a row's piece inside one slab would
    hold fewer than three entries on average (mean row length < 3 * number of slabs)."""
    slabs = -(-cols // (1 << SLAB_SHIFT))
    if rows > 0 and slabs >= 4 and nnz < 3 * slabs * rows:
        return SLAB_SHIFT + 1
    return SLAB_SHIFT


def slab_plan(rows: int, cols: int, row_ptr, col_idx, shift: int = SLAB_SHIFT):
    """The preprocessing result of the column-slabbed schedule (Sec. IV: a kernel may have a
    preprocessing step whose cost is amortised over the products; the format itself is this
    build's).  Column c belongs to slab c >> shift; there are S = ceil(cols / 2^shift) slabs.
    Row i is cut into S virtual rows, virtual row s * rows + i holding the entries of row i
    whose column lies in slab s, in the order they have in row i, and the entries are stored
    virtual row after virtual row -- all of slab 0 first, then slab 1, ...  Only the virtual
    rows that hold entries are kept, numbered 0 .. K - 1 in that order.  Returns
        n_slabs,
        rp_v  [S * rows + 1]  offsets of all virtual rows,
        perm  [nnz]           perm[p] = the CSR position of the p-th entry of the slabbed order,
        rp_z  [K + 1]         offsets of the kept virtual rows,
        rp_j  [rows + 1], p_idx [K]   row i's pieces are the kept rows p_idx[rp_j[i] : rp_j[i+1]],
                              in slab order,
    or None where the form does not apply: fewer than two slabs, S * rows >= 2^31, or a row
    whose columns do not ascend (then a virtual row would not be one piece of its row)."""
    rp = np.asarray(row_ptr, dtype=np.int64)
    nnz = int(rp[rows] - rp[0]) if rows > 0 else 0
    ci = np.asarray(col_idx[:nnz], dtype=np.int64)
    n_slabs = -(-int(cols) // (1 << shift))
    if rows <= 0 or n_slabs < 2 or n_slabs * rows >= 2 ** 31:
        return None
    lens = np.diff(rp[: rows + 1])
    row_of = np.repeat(np.arange(rows, dtype=np.int64), lens)
    if nnz > 1:
        descends = (ci[1:] < ci[:-1]) & (row_of[1:] == row_of[:-1])
        if np.any(descends):
            return None
    slab = ci >> shift
    perm = np.argsort(slab, kind="stable")           # slab-major; inside a slab the CSR order (row-major) stays
    v = slab[perm] * rows + row_of[perm]
    rp_v = np.zeros(n_slabs * rows + 1, dtype=np.int64)
    np.cumsum(np.bincount(v, minlength=n_slabs * rows), out=rp_v[1:])
    kept = np.flatnonzero(np.diff(rp_v) > 0)         # the virtual rows with entries, ascending
    rp_z = np.append(rp_v[kept], nnz)
    # row i's pieces: the kept rows whose number is i modulo rows, in slab (= ascending) order
    owner = kept % rows
    order = np.argsort(owner, kind="stable")
    rp_j = np.zeros(rows + 1, dtype=np.int64)
    np.cumsum(np.bincount(owner, minlength=rows), out=rp_j[1:])
    return {"n_slabs": n_slabs, "rp_v": rp_v, "perm": perm, "rp_z": rp_z, "rp_j": rp_j, "p_idx": order.astype(np.int64)}


def slab_spmv_python(rows, plan, col_idx, values, x):
    """y from the slabbed form, executed literally: the kept virtual rows' sums first, then,
    per row, the sum over its pieces in the listed order.  Exact arithmetic is the caller's
    business (use integer-valued data): pure Python, tiny inputs only."""
    rp_z, perm, rp_j, p_idx = plan["rp_z"], plan["perm"], plan["rp_j"], plan["p_idx"]
    yz = [0] * (len(rp_z) - 1)
    for j in range(len(yz)):
        for p in range(int(rp_z[j]), int(rp_z[j + 1])):
            k = int(perm[p])
            yz[j] += values[k] * x[int(col_idx[k])]
    return [sum(yz[int(p_idx[t])] for t in range(int(rp_j[i]), int(rp_j[i + 1]))) for i in range(rows)]


def csr_defects(rows: int, cols: int, nnz: int, row_ptr, col_idx):
    """(bad offsets, bad column indices) of a CSR matrix given as rows, cols, nnz and its
    two integer arrays.  An offset defect is: row_ptr[0] != 0 (one), row_ptr[rows] != nnz
    (one), and every i in [0, rows) with row_ptr[i + 1] < row_ptr[i] (one each).  A column
    defect is every k in [0, nnz) with col_idx[k] < 0 or col_idx[k] >= cols.  A matrix with
    (0, 0) is one every schedule may be run on: all offsets lie in [0, nnz], rows are
    contiguous ranges, and every gather stays inside x."""
    bad_rp = int(int(row_ptr[0]) != 0) + int(int(row_ptr[rows]) != nnz)
    for i in range(rows):
        if int(row_ptr[i + 1]) < int(row_ptr[i]):
            bad_rp += 1
    bad_ci = 0
    for k in range(nnz):
        c = int(col_idx[k])
        if c < 0 or c >= cols:
            bad_ci += 1
    return bad_rp, bad_ci
