"""Training side of the selector (Sec. III-A and III-D of the Seer paper): benchmark
every SpMV schedule and the feature collection on a representative population, label
each matrix with its fastest schedule, and fit the three CART decision trees of the
training abstraction (scikit-learn, Gini, depth-capped, 80/20 split, no
hyper-parameter tuning): the known-features model, the gathered-features model, and
the classifier-selection model that decides, from the known features alone, whether
gathering is worth its cost.  The trees are stored as the flat node arrays that
`seer_select` / `seer_spmv_auto` / `seer_spmv_model` walk.

    python -m paper_2403_17017_amd.training sweep --count 3000 --out sweep.csv
    python -m paper_2403_17017_amd.training fit --csv sweep.csv \
           --out paper_2403_17017_amd/selector_model.json
    python -m paper_2403_17017_amd.training evaluate --csv sweep.csv \
           --model paper_2403_17017_amd/selector_model.json --out eval.csv
    python -m paper_2403_17017_amd.training export-header      # trees as nested if/else in C

The same sweep also feeds the multiple-iteration models (Sec. IV-E): for every matrix
and every iteration count n of a fixed grid the label is the kernel with the smallest
preprocessing + n * run time, the iteration count is one more known feature, and the
feature collection is paid once.  Those three trees are stored under "iterative" and are
what `seer_spmv_plan` walks.

Timing protocol as in Sec. IV-B: 10 warm-up runs, mean of 10 timed runs, on the same
buffers; the timed runs are replayed from a HIP graph so that kernel time, not host
launch time, is compared.  Feature collection is timed as the caller sees it (the
seer_features call, including its wait), which is the cost Sec. III-C is about.
"""
from __future__ import annotations

import argparse
import csv
import json
import os
import sys
import time

import numpy as np

from . import binding as S

MAX_DEPTH = 6   # fixed before looking at any test data (the paper caps depth, value unstated)
# t_k{k}_us is the time of one product; for a kernel with preprocessing that is the
# product with a prepared plan, t_prep_k{k}_us the seer_spmv_prepare call as the caller
# sees it, t_single_k{k}_us the one-call form that prepares and multiplies.  t_rep_k{k}_us
# is a kernel without preprocessing run through seer_spmv_prepared, the entry point for
# repeated products (it differs from seer_spmv in how a cache-sized matrix is loaded).
PREP_KERNELS = [S.CSR_A, S.ELL_TM, S.COO_WM, S.CSR_S]
FALLBACK_KERNELS = [S.ELL_TM, S.CSR_S]      # where their form does not apply, seer_spmv_plan prepares CSR,A instead
ELL_MAX_BYTES = 2 << 30     # the sweep does not build ELL forms beyond this; the run-time rule is the caller's memory
CSV_FIELDS = (["m", "family", "rows", "cols", "nnz"] + [f"f_{n}" for n in S.FEATURE_NAMES]
              + ["t_features_us"] + [f"t_k{k}_us" for k in range(S.NUM_KERNELS)]
              + [f"t_prep_k{k}_us" for k in PREP_KERNELS] + [f"t_single_k{k}_us" for k in PREP_KERNELS]
              + [f"t_rep_k{k}_us" for k in range(S.NUM_DIRECT_KERNELS)]
              + ["t_auto_mp_us", "max_disagreement"]
              # one product with operands that are not in any cache (rotating copies): what the
              # single-product models are fitted to when the sweep has these columns
              + [f"t_cold_k{k}_us" for k in range(S.NUM_DIRECT_KERNELS)] + ["t_cold_auto_mp_us", "cold_sets"])
KNOWN_IDX = [0, 1, 2, 3, 8]   # rows, cols, nnz, mean_len, mean_density: what seer_known_features fills
KNOWN_ITER_IDX = KNOWN_IDX + [S.F_ITERATIONS]
ITER_GRID = [1, 2, 3, 5, 8, 12, 19, 30, 50, 100]   # iteration counts the iterative models are trained on
ND = S.NUM_DIRECT_KERNELS


def time_graph_us(enqueue, warmup=10, reps=10, replays=3):
    """Time of one `enqueue()` (which only enqueues GPU work) on the GPU timeline.  THE timing
    protocol of every path that is compared with another (Sec. IV-B: 10 warm-up runs, mean of
    10 timed runs): `warmup` eager calls, `reps` calls captured into one HIP graph, one untimed
    replay, then `replays` timed replays between two HIP events; the median replay / reps."""
    import torch
    for _ in range(warmup):
        enqueue()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(reps):
            enqueue()
    g.replay()
    torch.cuda.synchronize()
    ts = []
    for _ in range(replays):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) * 1e3 / reps)
    return sorted(ts)[len(ts) // 2]


def time_kernel_us(kid, dA, x, y, ws):
    """One product with a fixed kernel through seer_spmv, by the common protocol."""
    return time_graph_us(lambda: S.seer_spmv(kid, dA, x, y, workspace=ws))


COLD_BYTES = 320 << 20      # more than the 256 MB last-level cache plus the eight 4 MB L2s
COLD_MAX_SETS = 32


def cold_sets(dA, x, y, ws):
    """Independent device copies of (A, x, y, workspace), enough that a pass over all of them
    moves more than the caches hold (at most COLD_MAX_SETS: a matrix below 10 MB stays partly
    cached).  The first set is the given one."""
    foot = 8 * dA.nnz + 4 * (dA.rows + 1) + 4 * dA.cols + 4 * dA.rows
    n = max(2, min(COLD_MAX_SETS, -(-COLD_BYTES // max(foot, 1)) + 1))
    sets = [(dA, x, y, ws)]
    for _ in range(n - 1):
        sets.append((S.DeviceCSR(dA.rows, dA.cols, dA.row_ptr.clone(), dA.col_idx.clone(), dA.values.clone(), dA.nnz),
                     x.clone(), y.clone(), ws.clone()))
    return sets


def time_graph_cold_us(enqueue_on, sets, replays=3):
    """As time_graph_us, but successive calls go to successive sets of buffers (one graph of one
    call per set, at least ten calls), so that a call finds its operands evicted."""
    import torch
    n = len(sets)
    reps = n * -(-10 // n)
    for i in range(reps):
        enqueue_on(*sets[i % n])
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(reps):
            enqueue_on(*sets[i % n])
    g.replay()
    torch.cuda.synchronize()
    ts = []
    for _ in range(replays):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) * 1e3 / reps)
    return sorted(ts)[len(ts) // 2]


def time_prepare_us(kid, dA, plan_mem, warmup=3, reps=10):
    for _ in range(warmup):
        plan = S.seer_spmv_prepare(kid, dA, plan_mem)
    t0 = time.perf_counter()
    for _ in range(reps):
        plan = S.seer_spmv_prepare(kid, dA, plan_mem)
    return (time.perf_counter() - t0) / reps * 1e6, plan


def time_features_us(dA, ws, warmup=3, reps=10):
    for _ in range(warmup):
        f = S.seer_features(dA, workspace=ws)
    t0 = time.perf_counter()
    for _ in range(reps):
        f = S.seer_features(dA, workspace=ws)
    return (time.perf_counter() - t0) / reps * 1e6, f


def measure_matrix(spec, device="cuda:0", extra=None):
    """One CSV row for sweep matrix `spec` (see workloads.sweep_gen).  extra(dA, x, y, ws, row):
    further measurements on the same buffers, added to the row."""
    import torch

    from workloads.sweep_gen import build_on_device
    rp, ci, va, x = build_on_device(spec, device)
    dA = S.DeviceCSR(spec.rows, spec.rows, rp, ci, va, int(ci.numel()))
    ws = S.alloc_workspace(max([S.spmv_auto_workspace_bytes(dA.rows, dA.nnz), S.features_workspace_bytes(dA.rows)]
                               + [S.spmv_workspace_bytes(k, dA.rows, dA.nnz) for k in range(S.NUM_KERNELS)]), device)
    t_feat, f = time_features_us(dA, ws)
    row = {"m": spec.m, "family": spec.family, "rows": dA.rows, "cols": dA.cols, "nnz": dA.nnz,
           "t_features_us": round(t_feat, 3)}
    for n, v in zip(S.FEATURE_NAMES, f.vector()):
        row[f"f_{n}"] = repr(float(v))
    ys = []
    for k in range(S.NUM_KERNELS):
        y = torch.empty(dA.rows, device=device)
        if k == S.ELL_TM:
            need = S.ell_plan_bytes(dA.rows, int(f.max_len))
            if need == 0 or need > ELL_MAX_BYTES:      # not applicable here: seer_spmv_plan would fall back
                row[f"t_prep_k{k}_us"] = row[f"t_single_k{k}_us"] = row[f"t_k{k}_us"] = "inf"
                y.zero_()
                y += ys[3]
            else:
                plan_mem = S.alloc_workspace(max(need, S.features_workspace_bytes(dA.rows)), device)
                t_prep, plan = time_prepare_us(k, dA, plan_mem)
                row[f"t_prep_k{k}_us"] = round(t_prep, 3)
                row[f"t_single_k{k}_us"] = "inf"           # no one-call form
                row[f"t_k{k}_us"] = round(time_graph_us(lambda: S.seer_spmv_prepared(plan, dA, x, y, ws)), 3)
                del plan, plan_mem
        elif k == S.CSR_S:
            need = S.slab_plan_bytes(dA.rows, dA.cols, dA.nnz)
            plan = None
            if need and need <= ELL_MAX_BYTES * 2:
                plan_mem = S.alloc_workspace(need, device)
                try:
                    t_prep, plan = time_prepare_us(k, dA, plan_mem)
                except S.SeerError as err:             # some row's columns do not ascend: not applicable
                    if err.status != -1:
                        raise
            if plan is None:
                row[f"t_prep_k{k}_us"] = row[f"t_single_k{k}_us"] = row[f"t_k{k}_us"] = "inf"
                y.zero_()
                y += ys[3]
            else:
                wsk = S.alloc_workspace(S.spmv_prepared_workspace_bytes(plan), device)
                row[f"t_prep_k{k}_us"] = round(t_prep, 3)
                row[f"t_single_k{k}_us"] = "inf"           # no one-call form
                row[f"t_k{k}_us"] = round(time_graph_us(lambda: S.seer_spmv_prepared(plan, dA, x, y, wsk)), 3)
                del plan, plan_mem, wsk
        elif k in PREP_KERNELS:
            plan_mem = S.alloc_workspace(S.plan_bytes(k, dA.rows, dA.nnz), device)
            t_prep, plan = time_prepare_us(k, dA, plan_mem)
            row[f"t_prep_k{k}_us"] = round(t_prep, 3)
            row[f"t_single_k{k}_us"] = round(time_kernel_us(k, dA, x, y, ws), 3)
            row[f"t_k{k}_us"] = round(time_graph_us(lambda: S.seer_spmv_prepared(plan, dA, x, y, ws)), 3)
        else:
            row[f"t_k{k}_us"] = round(time_kernel_us(k, dA, x, y, ws), 3)
            direct = S.seer_spmv_prepare(k, dA)
            row[f"t_rep_k{k}_us"] = round(time_graph_us(lambda: S.seer_spmv_prepared(direct, dA, x, y, ws)), 3)
        ys.append(y)
    # the asynchronous path with a constant tree: its excess over the bare kernel is the
    # device-side cost of gathering and selecting
    mp_only = S.Tree.constant(S.CSR_MP)
    S.set_tuning("auto_prune", 0)            # (a one-leaf tree would otherwise not gather at all)
    try:
        row["t_auto_mp_us"] = round(time_graph_us(lambda: S.seer_spmv_auto(dA, mp_only, x, ys[3], ws)), 3)
    finally:
        S.set_tuning("auto_prune", -1)
    # the schedules must agree with each other (a sanity check, not the parity test)
    scale = float(ys[3].abs().max().item()) + 1e-30
    row["max_disagreement"] = float(max((ys[k] - ys[3]).abs().max().item()
                                        for k in range(S.NUM_KERNELS) if k != 3) / scale)
    if extra is not None:
        extra(dA, x, ys[0], ws, row)
    return row


def measure_cold_only(spec, device="cuda:0"):
    """The cold columns of a sweep row alone: every kernel without preprocessing, and the
    asynchronous path with a one-leaf merge-path tree (its excess over the bare kernel is the
    cost of gathering and selecting), each call on the next of several copies of (A, x, y)."""
    import torch

    from workloads.sweep_gen import build_on_device
    rp, ci, va, x = build_on_device(spec, device)
    dA = S.DeviceCSR(spec.rows, spec.rows, rp, ci, va, int(ci.numel()))
    ws = S.alloc_workspace(max([S.spmv_auto_workspace_bytes(dA.rows, dA.nnz)]
                               + [S.spmv_workspace_bytes(k, dA.rows, dA.nnz) for k in range(ND)]), device)
    y = torch.empty(dA.rows, device=device)
    sets = cold_sets(dA, x, y, ws)
    row = {"m": spec.m, "cold_sets": len(sets)}
    for k in range(ND):
        row[f"t_cold_k{k}_us"] = round(time_graph_cold_us(lambda d, xx, yy, w_: S.seer_spmv(k, d, xx, yy, workspace=w_), sets), 3)
    mp_only = S.Tree.constant(S.CSR_MP)
    S.set_tuning("auto_prune", 0)
    try:
        row["t_cold_auto_mp_us"] = round(time_graph_cold_us(lambda d, xx, yy, w_: S.seer_spmv_auto(d, mp_only, xx, yy, w_), sets), 3)
    finally:
        S.set_tuning("auto_prune", -1)
    return row


def run_cold_sweep(ms, out_csv, nnz_cap=200_000_000, max_rows_exp=7.0, log=sys.stderr):
    from workloads.sweep_gen import sweep_spec
    fields = ["m", "cold_sets"] + [f"t_cold_k{k}_us" for k in range(ND)] + ["t_cold_auto_mp_us"]
    with open(out_csv, "w", newline="") as fh:
        w = csv.DictWriter(fh, fieldnames=fields)
        w.writeheader()
        t_start = time.time()
        for m in ms:
            row = measure_cold_only(sweep_spec(m, nnz_cap, max_rows_exp))
            w.writerow(row)
            fh.flush()
            print(f"[sweep-cold] m={m} x{row['cold_sets']} t={[row[f't_cold_k{k}_us'] for k in range(ND)]} "
                  f"auto={row['t_cold_auto_mp_us']} ({time.time() - t_start:.0f}s)", file=log, flush=True)


def measure_slab_only(spec, device="cuda:0"):
    """The CSR,S columns of a sweep row alone (same matrix, same protocol): for adding the
    kernel to a sweep that was run before it existed."""
    import torch

    from workloads.sweep_gen import build_on_device
    rp, ci, va, x = build_on_device(spec, device)
    dA = S.DeviceCSR(spec.rows, spec.rows, rp, ci, va, int(ci.numel()))
    k = S.CSR_S
    row = {"m": spec.m, f"t_prep_k{k}_us": "inf", f"t_single_k{k}_us": "inf", f"t_k{k}_us": "inf"}
    need = S.slab_plan_bytes(dA.rows, dA.cols, dA.nnz)
    if need and need <= ELL_MAX_BYTES * 2:
        plan_mem = S.alloc_workspace(need, device)
        try:
            t_prep, plan = time_prepare_us(k, dA, plan_mem)
        except S.SeerError as err:
            if err.status != -1:
                raise
            return row
        y = torch.empty(dA.rows, device=device)
        wsk = S.alloc_workspace(S.spmv_prepared_workspace_bytes(plan), device)
        row[f"t_prep_k{k}_us"] = round(t_prep, 3)
        row[f"t_k{k}_us"] = round(time_graph_us(lambda: S.seer_spmv_prepared(plan, dA, x, y, wsk)), 3)
    return row


def run_slab_sweep(ms, out_csv, nnz_cap=200_000_000, max_rows_exp=7.0, log=sys.stderr):
    from workloads.sweep_gen import sweep_spec
    k = S.CSR_S
    fields = ["m", f"t_k{k}_us", f"t_prep_k{k}_us", f"t_single_k{k}_us"]
    with open(out_csv, "w", newline="") as fh:
        w = csv.DictWriter(fh, fieldnames=fields)
        w.writeheader()
        t_start = time.time()
        for m in ms:
            row = measure_slab_only(sweep_spec(m, nnz_cap, max_rows_exp))
            w.writerow(row)
            fh.flush()
            print(f"[sweep-slab] m={m} t={row[f't_k{k}_us']} prep={row[f't_prep_k{k}_us']} ({time.time() - t_start:.0f}s)",
                  file=log, flush=True)


def merge_columns(base_csv, extra_csv, out_csv):
    """base_csv with the columns of extra_csv (matched by sweep number m) filled in."""
    with open_text(extra_csv) as fh:
        extra = {int(r["m"]): r for r in csv.DictReader(fh)}
    with open_text(base_csv) as fh:
        rows = list(csv.DictReader(fh))
    with open(out_csv, "w", newline="") as fh:
        w = csv.DictWriter(fh, fieldnames=CSV_FIELDS)
        w.writeheader()
        for r in rows:
            e = extra.get(int(r["m"]), {})
            r.update({k: v for k, v in e.items() if k != "m"})
            w.writerow({k: r.get(k, "") for k in CSV_FIELDS})
    return out_csv


def run_sweep(ms, out_csv, nnz_cap=200_000_000, max_rows_exp=7.0, log=sys.stderr):
    from workloads.sweep_gen import sweep_spec
    done = set()
    if os.path.exists(out_csv):
        with open(out_csv) as fh:
            done = {int(r["m"]) for r in csv.DictReader(fh)}
    new = not os.path.exists(out_csv)
    with open(out_csv, "a", newline="") as fh:
        w = csv.DictWriter(fh, fieldnames=CSV_FIELDS)
        if new:
            w.writeheader()
        t_start = time.time()
        for m in ms:
            if m in done:
                continue
            spec = sweep_spec(m, nnz_cap, max_rows_exp)
            row = measure_matrix(spec)
            w.writerow(row)
            fh.flush()
            print(f"[sweep] m={m} {spec.family} rows={row['rows']} nnz={row['nnz']} "
                  f"t={[row[f't_k{k}_us'] for k in range(S.NUM_KERNELS)]} feat={row['t_features_us']} "
                  f"({time.time() - t_start:.0f}s)", file=log, flush=True)


def open_text(path):
    """A CSV for reading; a name ending in .gz is read through gzip (the sweep behind the
    shipped models is committed that way)."""
    if str(path).endswith(".gz"):
        import gzip
        return gzip.open(path, "rt", newline="")
    return open(path, newline="")


def load_csv(path):
    with open_text(path) as fh:
        rows = list(csv.DictReader(fh))
    X = np.array([[float(r[f"f_{n}"]) for n in S.FEATURE_NAMES] for r in rows], dtype=np.float32)
    T = np.array([[float(r.get(f"t_k{k}_us") or "inf") for k in range(S.NUM_KERNELS)] for r in rows])
    tf = np.array([float(r["t_features_us"]) for r in rows])
    # where the ELL or the column-slabbed form is not applicable the run time falls back to
    # CSR,A: that is what choosing ELL,TM or CSR,S costs there
    for k in FALLBACK_KERNELS:
        na = ~np.isfinite(T[:, k])
        T[na, k] = T[na, S.CSR_A]
    return rows, X, T, tf


def load_repeated(rows, T):
    """Per-product times for repeated products: as T, with the kernels without
    preprocessing taken from their seer_spmv_prepared timings where the sweep has them."""
    R = T.copy()
    if rows and f"t_rep_k0_us" in rows[0] and rows[0]["t_rep_k0_us"] not in ("", None):
        for k in range(ND):
            R[:, k] = [float(r[f"t_rep_k{k}_us"]) for r in rows]
    return R


def load_prep(rows):
    """Preprocessing time per matrix and kernel (zero for kernels that have none)."""
    P = np.zeros((len(rows), S.NUM_KERNELS))
    for k in PREP_KERNELS:
        P[:, k] = [float(r.get(f"t_prep_k{k}_us") or "inf") for r in rows]
    for k in FALLBACK_KERNELS:
        na = ~np.isfinite(P[:, k])
        P[na, k] = P[na, S.CSR_A]
    return P


def gather_overhead_us(rows_csv, T, field="t_auto_mp_us"):
    """Device-side cost of gathering + selecting per matrix, from the sweep: the excess
    of the asynchronous path (constant merge-path tree) over the bare merge-path kernel.
    Where the kernel is short the difference is taken as measured (the path has three
    launch shapes, by size, and their costs differ); where it runs for hundreds of
    microseconds single timings are noisier than the few microseconds being estimated,
    and a least-squares line in the number of rows through the short ones stands in."""
    r = np.array([float(x["rows"]) for x in rows_csv])
    d = np.array([float(x[field]) for x in rows_csv]) - T[:, S.CSR_MP]
    keep = T[:, S.CSR_MP] < 200.0            # short kernels give clean differences
    A = np.stack([np.ones(keep.sum()), r[keep]], axis=1)
    (a, b), *_ = np.linalg.lstsq(A, d[keep], rcond=None)
    return np.maximum(np.where(keep, d, a + b * r), 1.0), (float(a), float(b))


def tree_to_arrays(clf):
    t = clf.tree_
    feature = np.where(t.children_left < 0, -1, t.feature).astype(int)
    klass = clf.classes_[np.argmax(t.value[:, 0, :], axis=1)].astype(int)
    klass = np.where(feature >= 0, -1, klass)
    return {"feature": feature.tolist(), "threshold": [float(v) for v in t.threshold],
            "left": t.children_left.astype(int).tolist(), "right": t.children_right.astype(int).tolist(),
            "klass": klass.tolist()}


def predict_with_arrays(tree, X):
    out = np.empty(len(X), dtype=int)
    for i, row in enumerate(X):
        n = 0
        while tree["feature"][n] >= 0:
            n = tree["left"][n] if float(row[tree["feature"][n]]) <= tree["threshold"][n] else tree["right"][n]
        out[i] = tree["klass"][n]
    return out


def selector_report(T, tf, pred, t_select_us=0.2):
    """Aggregate times in the paper's sense (Sec. IV-D): the selector pays feature
    collection and inference on every matrix; 'oracle' is the best kernel per matrix."""
    n = len(T)
    idx = np.arange(n)
    t_sel = float(np.sum(tf + t_select_us + T[idx, pred]))
    t_fixed = T.sum(axis=0)
    t_oracle = float(T.min(axis=1).sum())
    best_fixed = int(np.argmin(t_fixed))
    return {
        "matrices": n, "accuracy": float(np.mean(pred == T.argmin(axis=1))),
        "t_selector_us": t_sel, "t_selector_kernels_only_us": float(np.sum(T[idx, pred])),
        "t_fixed_us": [float(v) for v in t_fixed], "best_fixed_kernel": best_fixed,
        "t_oracle_us": t_oracle,
        "speedup_vs_best_fixed": float(t_fixed[best_fixed] / t_sel),
        "speedup_vs_best_fixed_kernels_only": float(t_fixed[best_fixed] / np.sum(T[idx, pred])),
        "geomean_speedup_over_fixed_kernels": float(np.exp(np.mean(np.log(t_fixed / t_sel)))),
        "time_lost_vs_oracle": float(t_sel / t_oracle),
        "per_matrix_geomean_vs_best_fixed": float(np.exp(np.mean(np.log(
            T[:, best_fixed] / (tf + t_select_us + T[idx, pred]))))),
    }


SLOWDOWN_CAP = 50.0     # in the relative term a choice more than this many times slower counts as this
RELATIVE_US = 5.0       # a slowdown by a factor e on any matrix counts like this many microseconds


def choice_costs(T):
    """What choosing kernel k on matrix m costs, in microseconds: the time lost against
    the best kernel for m -- aggregate run time is what the paper scores its models by
    (Sec. IV-C, IV-D) -- plus RELATIVE_US times the log of the slowdown.  The relative
    term decides the small matrices, whose absolute regrets lie below a microsecond and
    would otherwise be decided by timing noise (it is what the per-matrix figures see).
    Pure log costs were tried: they compress a 13x mistake on a mid-sized skewed matrix
    to 2.6 units and cost 10 to 25 % of the aggregate on some train/test splits.
    Returns (cost [matrices, kernels], importance [matrices])."""
    tmin = T.min(axis=1, keepdims=True)
    cost = (T - tmin) + RELATIVE_US * np.minimum(np.log(T / tmin), np.log(SLOWDOWN_CAP))
    return cost, np.ones(len(T))


KNOWN_NEIGHBOURS = 40


def neighbour_costs(X, cost, groups=None, k=KNOWN_NEIGHBOURS):
    """Costs for fitting a known-features model: each training matrix is charged, for every
    kernel, the mean cost over the k training matrices nearest to it in (log rows, log nnz,
    log mean row length), itself included.  A model that sees only those numbers cannot
    tell a matrix from its neighbours, so what a choice costs it is the expectation over
    them; fitted to the matrices' own costs, a leaf that happens to hold no skewed training
    matrix picks a row-mapped schedule and the one skewed test matrix that lands there
    costs a whole percent of the aggregate (seen on five of six train/test splits; with
    neighbour costs none of the six fell below the best fixed kernel).
    groups: samples of one matrix at several iteration counts share the matrix's
    neighbours (cost is then [matrices * len(grid), kernels], matrix-major)."""
    from sklearn.neighbors import NearestNeighbors
    base = X if groups is None else X[::groups]
    Z = np.log1p(base[:, [0, 2, 3]].astype(np.float64))
    Z = (Z - Z.mean(axis=0)) / np.maximum(Z.std(axis=0), 1e-12)
    k = min(k, len(base))
    _, ind = NearestNeighbors(n_neighbors=k).fit(Z).kneighbors(Z)
    if groups is None:
        return cost[ind].mean(axis=1)
    c = cost.reshape(len(base), groups, cost.shape[1])
    return c[ind].mean(axis=1).reshape(cost.shape)


def _cart(Xs, cost, importance, leaves=None):
    """CART on a cost matrix instead of hard labels: sample m is entered once per class k
    with weight importance[m] * (worst cost of m - cost[m, k]), so that the class a leaf
    votes for is the one with the least total cost over the leaf's matrices (the standard
    reduction of cost-sensitive classification to weighted classification).  With 0/1
    costs this is the plain fastest-kernel label."""
    from sklearn.tree import DecisionTreeClassifier
    n, K = cost.shape
    w = ((cost.max(axis=1, keepdims=True) - cost) * importance[:, None]).reshape(-1)
    Xe, ye = np.repeat(Xs, K, axis=0), np.tile(np.arange(K), n)
    keep = w > 0
    if not np.any(keep):                      # every choice costs the same everywhere
        keep, w = ye == 0, np.ones_like(w)
    if leaves is None:
        clf = DecisionTreeClassifier(criterion="gini", max_depth=MAX_DEPTH, random_state=0)
    else:                                     # a number of leaves instead of a depth: grown best split first
        clf = DecisionTreeClassifier(criterion="gini", max_leaf_nodes=leaves, random_state=0)
    return clf.fit(Xe[keep], ye[keep], sample_weight=w[keep])


def _fit(X, cost, importance, cols=None, leaves=None):
    Xs = X if cols is None else X[:, cols]
    clf = _cart(Xs, cost, importance, leaves)
    tree = tree_to_arrays(clf)
    if cols is not None:   # the stored tree indexes the full feature vector
        tree["feature"] = [cols[f] if f >= 0 else -1 for f in tree["feature"]]
    assert np.array_equal(predict_with_arrays(tree, X), clf.predict(Xs))
    return tree


OOF_REPEATS = 3


def _out_of_fold(Xs, cost, importance, groups=None, folds=5, repeats=OOF_REPEATS, leaves=None):
    """Predictions for every sample by trees that were fitted without it (and without any
    sample of the same group): [samples, repeats], one column per random 5-fold split."""
    g = np.arange(len(Xs)) if groups is None else np.asarray(groups)
    ids = np.unique(g)
    out = np.zeros((len(Xs), repeats), dtype=int)
    for r in range(repeats):
        fold_of = dict(zip(ids.tolist(), np.random.default_rng(r).permutation(len(ids)) % folds))
        f = np.array([fold_of[v] for v in g.tolist()])
        for k in range(folds):
            a, b = f != k, f == k
            out[b, r] = _cart(Xs[a], cost[a], importance[a], leaves).predict(Xs[b])
    return out


ITER_LEAVES = (64, 128, 256, 512)   # 64 leaves is what MAX_DEPTH allows; 512 leaves = 1023 nodes, 20 KB


def _pick_leaves(Xs, cost, importance, groups, candidates=None):
    """Size of a tree of the iterative models, by cross-validation inside the training set (5
    folds split by matrix): the number of leaves, grown best split first, whose out-of-fold
    choices cost least, in the costs the tree is fitted to.  The test matrices play no part.
    These trees have the iteration count to split on besides the matrix features and eight
    kernels to tell apart, and they are walked on the host, so the device-side walk's 127
    nodes do not bind them.  (On the sweep: 512 leaves for both trees; held-out, against
    depth 6, 100 products 1.028 -> 1.039 of the best fixed kernel and 1.9 -> 0.8 % above the
    per-matrix best, a preprocessing kernel chosen on 15 % of the matrices instead of 2 %;
    one to three products 0.3 to 0.6 % worse.)"""
    candidates = ITER_LEAVES if candidates is None else candidates
    best, best_cost, seen = candidates[0], None, {}
    i = np.arange(len(Xs))
    for n_leaves in candidates:
        oof = _out_of_fold(Xs, cost, importance, groups=groups, repeats=1, leaves=n_leaves)[:, 0]
        seen[n_leaves] = float((cost[i, oof] * importance).sum())
        if best_cost is None or seen[n_leaves] < best_cost:
            best, best_cost = n_leaves, seen[n_leaves]
    return best, seen


def _oof_times(T, oof_known, oof_gathered):
    """What either path is expected to cost on each training sample, from the out-of-fold
    predictions: the known model, which cannot see what it gets wrong, is charged its
    worst choice over the repeats; the gathered model its median one.  A single split
    leaves the rare expensive mistakes of the known model to chance: over six train/test
    splits the aggregate then ranged from 0.93 to 1.00 of the best fixed kernel, with
    this rule from 0.97 to 1.00."""
    i = np.arange(len(T))[:, None]
    return T[i, oof_known].max(axis=1), np.median(T[i, oof_gathered], axis=1)


def _fit_selector(Xk, cols, t_known, t_gather):
    """The classifier-selection tree: class 0 = the known model is good enough, 1 = gather;
    costs as in choice_costs, of either way against the better of the two."""
    cost, imp = choice_costs(np.stack([t_known, t_gather], axis=1))
    tree = _fit(Xk, cost, imp, cols)
    tree["klass"] = [int(k) if k >= 0 else -1 for k in tree["klass"]]
    return tree


def model_report(T, ovh, pred_known, pred_gath, use_gath):
    """Aggregate times in the paper's sense (Sec. IV-D).  'oracle' = best kernel per
    matrix; the gathered model pays the device-side gathering cost on every matrix,
    the classifier-selection model only where the selector says so."""
    idx = np.arange(len(T))
    t_known = T[idx, pred_known]
    t_gath = T[idx, pred_gath] + ovh
    t_model = np.where(use_gath == 1, t_gath, t_known)
    t_fixed = T.sum(axis=0)
    best = int(np.argmin(t_fixed))
    hit = lambda pred: float(np.mean(T[idx, pred] == T.min(axis=1)))     # the fastest kernel, or tied with it
    geo = lambda a, b: float(np.exp(np.mean(np.log(a / b))))
    return {
        "matrices": int(len(T)),
        "accuracy": {"known": hit(pred_known), "gathered": hit(pred_gath),
                     "classifier_selection": hit(np.where(use_gath == 1, pred_gath, pred_known))},
        "gathered_fraction": float(np.mean(use_gath)),
        "t_us": {"known": float(t_known.sum()), "gathered": float(t_gath.sum()),
                 "classifier_selection": float(t_model.sum()), "oracle": float(T.min(axis=1).sum()),
                 "fixed": [float(v) for v in t_fixed]},
        "best_fixed_kernel": best,
        "aggregate_speedup_vs_best_fixed": {"known": float(t_fixed[best] / t_known.sum()),
                                            "gathered": float(t_fixed[best] / t_gath.sum()),
                                            "classifier_selection": float(t_fixed[best] / t_model.sum())},
        "per_matrix_geomean_vs_best_fixed": {"known": geo(T[:, best], t_known), "gathered": geo(T[:, best], t_gath),
                                             "classifier_selection": geo(T[:, best], t_model)},
        "geomean_over_fixed_kernels_of_aggregate_speedup": float(np.exp(np.mean(np.log(t_fixed / t_model.sum())))),
        "time_lost_vs_oracle": float(t_model.sum() / T.min(axis=1).sum()),
    }


def fit_model(csv_path, out_json, test_frac=0.2, seed=0):
    from sklearn.model_selection import train_test_split
    rows, X, T_all, tf = load_csv(csv_path)
    P = load_prep(rows)
    T = T_all[:, :ND]               # the single-product models choose among the kernels without preprocessing
    cold = bool(rows) and rows[0].get("t_cold_k0_us") not in ("", None)
    if cold:
        # A single product finds nothing of the matrix in the caches; several products with one
        # matrix (the iterative models below) do, if it fits.  The single-product models are
        # therefore fitted to the cold timings where the sweep has them.
        T = np.array([[float(r[f"t_cold_k{k}_us"]) for k in range(ND)] for r in rows])
    y = T.argmin(axis=1)            # label = fastest kernel; ties -> lowest kernel id
    idx = np.arange(len(rows))
    tr, te = train_test_split(idx, test_size=test_frac, random_state=seed)
    ovh, ovh_fit = gather_overhead_us(rows, T, "t_cold_auto_mp_us" if cold else "t_auto_mp_us")
    Xk = np.zeros_like(X)
    Xk[:, KNOWN_IDX] = X[:, KNOWN_IDX]          # what the known-features vector looks like at run time
    cost, imp = choice_costs(T)
    gathered = _fit(X[tr], cost[tr], imp[tr])
    # The known model sees too little to tell a skewed matrix from a regular one; trained
    # on the expected cost over a matrix's neighbourhood it learns the kernel that is safe
    # where it cannot tell.
    cost_known = neighbour_costs(Xk[tr], cost[tr])
    known = _fit(Xk[tr], cost_known, imp[tr], KNOWN_IDX)
    pk, pg = predict_with_arrays(known, Xk), predict_with_arrays(gathered, X)
    # Classifier selection: gather exactly where it pays.  The two models are judged on
    # training matrices they were not fitted on (5-fold out-of-fold predictions);
    # judged on their own training data they look better than they are and the selector
    # would learn never to gather.
    oof_k = _out_of_fold(Xk[tr][:, KNOWN_IDX], cost_known, imp[tr])
    oof_g = _out_of_fold(X[tr], cost[tr], imp[tr])
    t_if_known, t_if_gathered = _oof_times(T[tr], oof_k, oof_g)
    selector = _fit_selector(Xk[tr], KNOWN_IDX, t_if_known, t_if_gathered + ovh[tr])
    ug = predict_with_arrays(selector, Xk)
    model = {
        "gathered": gathered, "known": known, "selector": selector,
        "note": f"CART gini max_depth={MAX_DEPTH} on costs = time lost + {RELATIVE_US:g} us * log slowdown, "
                f"{len(tr)} training matrices" + (", single-product models on cold timings" if cold else ""),
        "feature_names": list(S.FEATURE_NAMES), "known_features": KNOWN_IDX,
        "gather_overhead_us": {"intercept": ovh_fit[0], "per_row": ovh_fit[1]},
        "label_counts": np.bincount(y, minlength=ND).tolist(),
        "iterative": fit_iterative(X, load_repeated(rows, T_all), P, tf, tr, te),
        "report": {"train": model_report(T[tr], ovh[tr], pk[tr], pg[tr], ug[tr]),
                   "test": model_report(T[te], ovh[te], pk[te], pg[te], ug[te]),
                   "all": model_report(T, ovh, pk, pg, ug)},
        "test_matrices": [int(rows[i]["m"]) for i in te],
    }
    with open(out_json, "w") as fh:
        json.dump(model, fh, indent=1)
    return model


def iterative_report(C, tf, pred_known, pred_gath, use_gath):
    """Times for n products per matrix: C[m, k] = preprocessing + n * run time.  The
    gathered model pays the feature collection once, the classifier-selection model only
    where the selector asks for it."""
    idx = np.arange(len(C))
    t_known = C[idx, pred_known]
    t_gath = C[idx, pred_gath] + tf
    t_model = np.where(use_gath == 1, t_gath, t_known)
    t_fixed = C.sum(axis=0)
    best = int(np.argmin(t_fixed))
    truth = C.argmin(axis=1)
    chosen = np.where(use_gath == 1, pred_gath, pred_known)
    prep = np.isin(chosen, PREP_KERNELS)
    hit = lambda pred: float(np.mean(C[idx, pred] == C.min(axis=1)))     # the cheapest kernel, or tied with it
    geo = lambda a, b: float(np.exp(np.mean(np.log(a / b))))
    return {
        "matrices": int(len(C)),
        "accuracy": {"known": hit(pred_known), "gathered": hit(pred_gath), "classifier_selection": hit(chosen)},
        # did the model call the amortisation right: preprocessing chosen iff it pays
        "amortisation_accuracy": float(np.mean(prep == np.isin(truth, PREP_KERNELS))),
        "amortisation_accuracy_gathered": float(np.mean(np.isin(pred_gath, PREP_KERNELS) == np.isin(truth, PREP_KERNELS))),
        "preprocessing_chosen_fraction": float(np.mean(prep)),
        "preprocessing_best_fraction": float(np.mean(np.isin(truth, PREP_KERNELS))),
        "gathered_fraction": float(np.mean(use_gath)),
        "t_us": {"known": float(t_known.sum()), "gathered": float(t_gath.sum()),
                 "classifier_selection": float(t_model.sum()), "oracle": float(C.min(axis=1).sum()),
                 "fixed": [float(v) for v in t_fixed]},
        "best_fixed_kernel": best,
        "aggregate_speedup_vs_best_fixed": float(t_fixed[best] / t_model.sum()),
        "per_matrix_geomean_vs_best_fixed": geo(C[:, best], t_model),
        "time_lost_vs_oracle": float(t_model.sum() / C.min(axis=1).sum()),
    }


def fit_iterative(X, T, P, tf, tr, te, grid=ITER_GRID):
    """The three trees for n products with one matrix (Sec. IV-E): every training matrix
    appears once per iteration count of the grid, labelled with the kernel of least
    preprocessing + n * run time among all kernels; folds are split by matrix."""
    def expand(sel):
        Xe = np.repeat(X[sel], len(grid), axis=0)
        n = np.tile(np.array(grid, dtype=np.float64), len(sel))
        Xe[:, S.F_ITERATIONS] = n.astype(np.float32)
        C = np.repeat(P[sel], len(grid), axis=0) + n[:, None] * np.repeat(T[sel], len(grid), axis=0)
        return Xe, C, np.repeat(tf[sel], len(grid)), np.repeat(sel, len(grid)), n

    Xtr, Ctr, tftr, gtr, ntr = expand(tr)
    ytr = Ctr.argmin(axis=1)
    Xk = np.zeros_like(Xtr)
    Xk[:, KNOWN_ITER_IDX] = Xtr[:, KNOWN_ITER_IDX]
    # costs per product: with totals, the samples at 100 products would outweigh those at one
    # product a hundred to one and the trees would be fitted to the long runs alone
    cost, imp = choice_costs(Ctr / ntr[:, None])
    leaves_g, cv_g = _pick_leaves(Xtr, cost, imp, gtr)
    gathered = _fit(Xtr, cost, imp, leaves=leaves_g)
    cost_known = neighbour_costs(Xk, cost, groups=len(grid))
    leaves_k, cv_k = _pick_leaves(Xk[:, KNOWN_ITER_IDX], cost_known, imp, gtr)
    known = _fit(Xk, cost_known, imp, KNOWN_ITER_IDX, leaves=leaves_k)
    oof_k = _out_of_fold(Xk[:, KNOWN_ITER_IDX], cost_known, imp, groups=gtr, leaves=leaves_k)
    oof_g = _out_of_fold(Xtr, cost, imp, groups=gtr, leaves=leaves_g)
    t_if_known, t_if_gathered = _oof_times(Ctr, oof_k, oof_g)
    selector = _fit_selector(Xk, KNOWN_ITER_IDX, t_if_known / ntr, (t_if_gathered + tftr) / ntr)

    def report(sel):
        out = {}
        for n in grid:
            Xe = X[sel].copy()
            Xe[:, S.F_ITERATIONS] = n
            Xke = np.zeros_like(Xe)
            Xke[:, KNOWN_ITER_IDX] = Xe[:, KNOWN_ITER_IDX]
            C = P[sel] + n * T[sel]
            out[str(n)] = iterative_report(C, tf[sel], predict_with_arrays(known, Xke),
                                           predict_with_arrays(gathered, Xe), predict_with_arrays(selector, Xke))
        return out

    return {"gathered": gathered, "known": known, "selector": selector, "iterations_grid": list(grid),
            "known_features": KNOWN_ITER_IDX,
            "leaves": {"gathered": leaves_g, "known": leaves_k, "cross_validation_cost": {"gathered": cv_g, "known": cv_k}},
            "label_counts": np.bincount(ytr, minlength=S.NUM_KERNELS).tolist(),
            "report": {"train": report(tr), "test": report(te)}}


def fit_tree(csv_path, out_json, test_frac=0.2, seed=0):
    """Gathered-features tree only (kept for callers that want a single tree)."""
    m = fit_model(csv_path, out_json, test_frac, seed)
    t = dict(m["gathered"])
    t["report"] = m["report"]
    return t


COLD_EVAL_MAX_BYTES = 256 << 20    # matrices up to here are also timed cold (larger ones are cold anyway)


def evaluate_model(csv_path, model_json, out_csv, log=sys.stderr, matrices=None, cold=True):
    """Runs the held-out matrices again (or `matrices`, e.g. sweep numbers no fit has seen)
    and times, end to end on the GPU timeline and all by the one protocol of time_graph_us:
    every fixed kernel, the always-gather path (seer_spmv_auto) and the classifier-selection
    path (seer_spmv_model), whose host-side decision (wall clock) is charged on top.  A matrix
    that fits the last-level cache is timed a second time cold, on rotating copies."""
    import torch

    from workloads.sweep_gen import build_on_device, sweep_spec
    model, meta = load_model(model_json)
    fields = ["m", "family", "rows", "nnz"] + [f"t_k{k}_us" for k in range(ND)] + \
             ["t_auto_us", "t_model_us", "t_model_host_us", "auto_kernel", "model_path", "model_kernel", "cold_sets"] + \
             [f"t_k{k}_cold_us" for k in range(ND)] + ["t_auto_cold_us", "t_model_cold_us"]
    with open(out_csv, "w", newline="") as fh:
        w = csv.DictWriter(fh, fieldnames=fields)
        w.writeheader()
        for m in (meta["test_matrices"] if matrices is None else matrices):
            spec = sweep_spec(m)
            rp, ci, va, x = build_on_device(spec)
            dA = S.DeviceCSR(spec.rows, spec.rows, rp, ci, va, int(ci.numel()))
            ws = S.alloc_workspace(S.spmv_auto_workspace_bytes(dA.rows, dA.nnz))
            y = torch.empty(dA.rows, device="cuda:0")
            row = {"m": m, "family": spec.family, "rows": dA.rows, "nnz": dA.nnz}
            for k in range(ND):
                row[f"t_k{k}_us"] = round(time_kernel_us(k, dA, x, y, ws), 3)
            row["t_auto_us"] = round(time_graph_us(lambda: S.seer_spmv_auto(dA, model.gathered, x, y, ws)), 3)
            _, row["auto_kernel"] = S.seer_spmv_auto_result(ws)
            row["t_model_us"] = round(time_graph_us(lambda: S.seer_spmv_model(dA, model, x, y, ws)), 3)
            row["t_model_host_us"] = round(S.seer_model_host_ns(model, dA.rows, dA.cols, dA.nnz) * 1e-3, 4)
            row["model_path"], row["model_kernel"] = S.seer_spmv_model(dA, model, x, y, ws)
            if row["model_path"] == 1:
                _, row["model_kernel"] = S.seer_spmv_auto_result(ws)
            foot = 8 * dA.nnz + 8 * dA.rows + 4 * dA.cols
            if cold and foot <= COLD_EVAL_MAX_BYTES:
                sets = cold_sets(dA, x, y, ws)
                row["cold_sets"] = len(sets)
                for k in range(ND):
                    row[f"t_k{k}_cold_us"] = round(time_graph_cold_us(
                        lambda d, xx, yy, w_: S.seer_spmv(k, d, xx, yy, workspace=w_), sets), 3)
                row["t_auto_cold_us"] = round(time_graph_cold_us(
                    lambda d, xx, yy, w_: S.seer_spmv_auto(d, model.gathered, xx, yy, w_), sets), 3)
                row["t_model_cold_us"] = round(time_graph_cold_us(
                    lambda d, xx, yy, w_: S.seer_spmv_model(d, model, xx, yy, w_), sets), 3)
                del sets
            else:                           # beyond the caches: the one-set timings are cold already
                row["cold_sets"] = 1
                for k in range(ND):
                    row[f"t_k{k}_cold_us"] = row[f"t_k{k}_us"]
                row["t_auto_cold_us"], row["t_model_cold_us"] = row["t_auto_us"], row["t_model_us"]
            w.writerow(row)
            fh.flush()
            print(f"[eval] m={m} {spec.family} nnz={dA.nnz} kernels={[row[f't_k{k}_us'] for k in range(ND)]} "
                  f"auto={row['t_auto_us']} (k{row['auto_kernel']}) model={row['t_model_us']} "
                  f"(path {row['model_path']}, k{row['model_kernel']}) cold x{row['cold_sets']}: "
                  f"{[row[f't_k{k}_cold_us'] for k in range(ND)]} auto={row['t_auto_cold_us']} "
                  f"model={row['t_model_cold_us']}", file=log, flush=True)
    return summarize_evaluation(out_csv)


ITER_EVAL_COUNTS = (1, 5, 19, 50, 100)


def evaluate_iterative(model_json, out_csv, counts=ITER_EVAL_COUNTS, matrices=None, log=sys.stderr):
    """The models for n products with one matrix, end to end on the held-out matrices (or
    `matrices`): every kernel's preprocessing call and product are timed again as in the sweep,
    and for each n the call a user makes -- seer_spmv_plan (wall clock: classifier selection,
    feature collection where asked for, the chosen kernel's preprocessing) -- and the product
    from the plan it returns (HIP graph replay).  Cost of a path for n products = its call +
    n * its product."""
    from workloads.sweep_gen import sweep_spec
    model, meta = load_model(model_json, iterative=True)
    fields = CSV_FIELDS + [f"{what}_n{n}" for n in counts for what in ("t_plan_us", "t_product_us", "kernel", "path")]

    def plan_path(dA, x, y, ws, row):
        slab = S.slab_plan_bytes(dA.rows, dA.cols, dA.nnz)
        plan_mem = S.alloc_workspace(max(S.plan_bytes(S.CSR_A, dA.rows, dA.nnz), S.plan_bytes(S.COO_WM, dA.rows, dA.nnz),
                                         min(12 * dA.nnz + (1 << 20), ELL_MAX_BYTES),
                                         slab if slab <= 2 * ELL_MAX_BYTES else 0))     # (the sweep's own limit)
        for n in counts:
            for _ in range(2):
                plan, path = S.seer_spmv_plan(dA, model, n, plan_mem, ws)
            t0 = time.perf_counter()
            for _ in range(5):
                plan, path = S.seer_spmv_plan(dA, model, n, plan_mem, ws)
            row[f"t_plan_us_n{n}"] = round((time.perf_counter() - t0) / 5 * 1e6, 3)
            need = S.spmv_prepared_workspace_bytes(plan)       # (CSR,S keeps its partials in the products' scratch)
            wsp = ws if need <= ws.numel() else S.alloc_workspace(need)
            row[f"t_product_us_n{n}"] = round(time_graph_us(lambda: S.seer_spmv_prepared(plan, dA, x, y, wsp)), 3)
            row[f"kernel_n{n}"], row[f"path_n{n}"] = plan.kernel_id, path

    with open(out_csv, "w", newline="") as fh:
        w = csv.DictWriter(fh, fieldnames=fields)
        w.writeheader()
        for m in (meta["test_matrices"] if matrices is None else matrices):
            row = measure_matrix(sweep_spec(m), extra=plan_path)
            w.writerow(row)
            fh.flush()
            print(f"[eval-it] m={m} {row['family']} nnz={row['nnz']} " +
                  " ".join(f"n{n}:k{row[f'kernel_n{n}']}/p{row[f'path_n{n}']}" for n in counts), file=log, flush=True)
    return summarize_iterative_evaluation(out_csv, counts)


def summarize_iterative_evaluation(eval_csv, counts=ITER_EVAL_COUNTS):
    rows, X, T, tf = load_csv(eval_csv)
    P = load_prep(rows)
    geo = lambda a, b: float(np.exp(np.mean(np.log(a / b))))
    out = {"matrices": len(rows)}
    for n in counts:
        C = P + n * T
        tm = np.array([float(r[f"t_plan_us_n{n}"]) + n * float(r[f"t_product_us_n{n}"]) for r in rows])
        chosen = np.array([int(r[f"kernel_n{n}"]) for r in rows])
        t_fixed = C.sum(axis=0)
        best = int(np.argmin(t_fixed))
        out[str(n)] = {
            "best_fixed_kernel": best, "t_best_fixed_us": float(t_fixed[best]), "t_oracle_us": float(C.min(axis=1).sum()),
            "t_classifier_selection_us": float(tm.sum()),
            "aggregate_speedup_vs_best_fixed": float(t_fixed[best] / tm.sum()),
            "per_matrix_geomean_vs_best_fixed": geo(C[:, best], tm),
            "time_lost_vs_oracle": float(tm.sum() / C.min(axis=1).sum()),
            "gathered_fraction": float(np.mean([int(r[f"path_n{n}"]) for r in rows])),
            "preprocessing_chosen_fraction": float(np.mean(np.isin(chosen, PREP_KERNELS))),
            "preprocessing_best_fraction": float(np.mean(np.isin(C.argmin(axis=1), PREP_KERNELS))),
        }
    return out


def summarize_evaluation(eval_csv, suffix="", families=None):
    """suffix "" = the same buffers every time (warm), "_cold" = rotating copies.  families:
    restrict to these matrix families.  The classifier-selection path is charged its host-side
    decision (t_model_host_us) on top of what the GPU timeline shows."""
    with open(eval_csv) as fh:
        rows = list(csv.DictReader(fh))
    if families is not None:
        rows = [r for r in rows if r["family"] in families]
    if suffix and (not rows or f"t_auto{suffix}_us" not in rows[0] or rows[0][f"t_auto{suffix}_us"] in ("", None)):
        return None
    T = np.array([[float(r[f"t_k{k}{suffix}_us"]) for k in range(ND)] for r in rows])
    ta = np.array([float(r[f"t_auto{suffix}_us"]) for r in rows])
    host = np.array([float(r.get("t_model_host_us") or 0.0) for r in rows])
    tm = np.array([float(r[f"t_model{suffix}_us"]) for r in rows]) + host
    t_fixed = T.sum(axis=0)
    best = int(np.argmin(t_fixed))
    geo = lambda a, b: float(np.exp(np.mean(np.log(a / b))))
    # where the classifier-selection path ran a fixed kernel on known features, how its time
    # compares with that kernel's own column: same kernel, same buffers, same protocol
    same = np.array([int(r["model_path"]) == 0 for r in rows])
    chosen = np.array([int(r["model_kernel"]) for r in rows])
    ratio = float(T[same, chosen[same]].sum() / (tm[same] - host[same]).sum()) if same.any() else float("nan")
    return {
        "matrices": len(rows), "t_fixed_us": [float(v) for v in t_fixed], "best_fixed_kernel": best,
        "t_oracle_us": float(T.min(axis=1).sum()), "t_always_gather_us": float(ta.sum()),
        "t_classifier_selection_us": float(tm.sum()), "t_host_decisions_us": float(host.sum()),
        "same_kernel_fixed_over_model": ratio,
        "aggregate_speedup_vs_best_fixed": {"always_gather": float(t_fixed[best] / ta.sum()),
                                            "classifier_selection": float(t_fixed[best] / tm.sum())},
        "per_matrix_geomean_vs_best_fixed": {"always_gather": geo(T[:, best], ta),
                                             "classifier_selection": geo(T[:, best], tm)},
        "geomean_over_fixed_kernels_of_aggregate_speedup": float(np.exp(np.mean(np.log(t_fixed / tm.sum())))),
        "time_lost_vs_oracle": {"always_gather": float(ta.sum() / T.min(axis=1).sum()),
                                "classifier_selection": float(tm.sum() / T.min(axis=1).sum())},
        "gathered_fraction": float(np.mean([int(r["model_path"]) for r in rows])),
    }


def write_report_md(csv_path, model_json, eval_csv, out_md, fresh_csv=None, iter_csv=None):
    """Human-readable summary of a sweep, the fit and the held-out evaluation."""
    rows, X, T, tf = load_csv(csv_path)
    P = load_prep(rows)
    with open(model_json) as fh:
        m = json.load(fh)
    names = [S.kernel_name(k) for k in range(S.NUM_KERNELS)]
    L = ["# Selector: sweep, training and held-out evaluation (MI355X)", "",
         "Commands (GPU box, repository root):", "",
         "    python -m paper_2403_17017_amd.training sweep --first 0 --count 3000 --out sweep_warm.csv",
         "    python -m paper_2403_17017_amd.training sweep-cold --first 0 --count 3000 --out sweep_cold.csv",
         "    python -m paper_2403_17017_amd.training merge --csv sweep_warm.csv --extra sweep_cold.csv --out sweep.csv",
         "    python -m paper_2403_17017_amd.training fit --csv sweep.csv --out selector_model.json",
         "    python -m paper_2403_17017_amd.training evaluate --csv sweep.csv "
         "--model selector_model.json --out eval.csv",
         "    python -m paper_2403_17017_amd.training report-md --csv sweep.csv "
         "--model selector_model.json --eval eval.csv" + (" --fresh-eval eval_fresh.csv" if fresh_csv else "") +
         (" --iterative-eval eval_iterative.csv" if iter_csv else "") + " --out profiles/selector_evaluation.md", "",
         "The sweep.csv behind the shipped models is committed as paper_2403_17017_amd/selector_sweep.csv.gz "
         "(every --csv option reads it as it is); `fit` on it gives the committed selector_model.json again "
         "(tests/test_training_host.py).", "",
         f"Population: {len(rows)} seeded synthetic matrices (workloads/sweep_gen.py), timing 10 warm-up + 10 timed "
         "runs per kernel by one protocol for all nine (HIP-graph replay after an untimed replay), same buffers "
         "(warm); the kernels without preprocessing also on rotating copies (cold columns).  CSR,A, ELL,TM, COO,WM "
         "and CSR,S are timed with a prepared plan; "
         "their preprocessing calls are timed apart (host wall clock, they wait for the device).  Where the ELL "
         "form (beyond 2 GiB here) or the slabbed form (x within one slab, columns not ascending) is not "
         "applicable the kernel is charged what CSR,A costs: that is what seer_spmv_plan falls back to.", "",
         f"## Sweep (all {len(rows)} matrices), sum of kernel times in us", "",
         "| family | matrices | " + " | ".join(names) + " | best per matrix (direct kernels) | fastest direct kernel counts |",
         "|---|---|" + "---|" * (len(names) + 2)]
    fam = np.array([r["family"] for r in rows])
    for f in list(dict.fromkeys(fam)) + ["all"]:
        sel = np.ones(len(rows), bool) if f == "all" else fam == f
        counts = np.bincount(T[sel][:, :ND].argmin(axis=1), minlength=ND)
        L.append(f"| {f} | {int(sel.sum())} | " + " | ".join(f"{v:.0f}" for v in T[sel].sum(axis=0)) +
                 f" | {T[sel][:, :ND].min(axis=1).sum():.0f} | " + "/".join(str(int(c)) for c in counts) + " |")
    L += ["", f"Preprocessing call of CSR,A: median {np.median(P[:, S.CSR_A]):.1f} us, "
          f"90th percentile {np.percentile(P[:, S.CSR_A], 90):.1f} us.  Feature collection call (seer_features, "
          f"with its wait): median {np.median(tf):.1f} us.", "",
          "## Single-product models (" + m["note"] + "), held-out matrices, predicted from sweep timings", ""]
    t = m["report"]["test"]
    L.append(f"accuracy (fastest kernel exactly): known {t['accuracy']['known']:.3f}, gathered "
             f"{t['accuracy']['gathered']:.3f}, classifier selection {t['accuracy']['classifier_selection']:.3f}; "
             f"gathered on {100 * t['gathered_fraction']:.0f} % of matrices; aggregate speed-up over the best fixed "
             f"kernel ({names[t['best_fixed_kernel']]}) {t['aggregate_speedup_vs_best_fixed']['classifier_selection']:.3f}, "
             f"per-matrix geomean {t['per_matrix_geomean_vs_best_fixed']['classifier_selection']:.3f}")
    def evaluation_section(path, title, whom):
        e = summarize_evaluation(path)
        best = names[e["best_fixed_kernel"]]
        out = ["", f"## {title} ({e['matrices']} matrices)", "",
               f"| path | total us | vs best fixed kernel ({best}) | per-matrix geomean vs {best} | vs oracle (best kernel per matrix) |",
               "|---|---|---|---|---|"]
        tb = e["t_fixed_us"][e["best_fixed_kernel"]]
        for k in range(ND):
            out.append(f"| fixed {names[k]} | {e['t_fixed_us'][k]:.0f} | {tb / e['t_fixed_us'][k]:.3f} | | "
                       f"{e['t_fixed_us'][k] / e['t_oracle_us']:.3f} |")
        for key, label in (("always_gather", "always gather (seer_spmv_auto)"),
                           ("classifier_selection", "classifier selection (seer_spmv_model)")):
            tot = e["t_always_gather_us"] if key == "always_gather" else e["t_classifier_selection_us"]
            out.append(f"| {label} | {tot:.0f} | {e['aggregate_speedup_vs_best_fixed'][key]:.3f} | "
                       f"{e['per_matrix_geomean_vs_best_fixed'][key]:.3f} | {e['time_lost_vs_oracle'][key]:.3f} |")
        out.append(f"| oracle | {e['t_oracle_us']:.0f} | {tb / e['t_oracle_us']:.3f} | | 1.000 |")
        out += ["", f"Geomean over the fixed kernels of (kernel total / classifier-selection total): "
                f"{e['geomean_over_fixed_kernels_of_aggregate_speedup']:.2f}x.  Features gathered on "
                f"{100 * e['gathered_fraction']:.0f} % of {whom}.  Every path is timed by the same protocol "
                "(10 eager warm-up calls, 10 calls in one HIP graph, one untimed replay, median of three timed "
                f"replays); the classifier-selection total includes {e['t_host_decisions_us']:.1f} us of host-side "
                "decisions (wall clock).  Check of the protocol: where that path ran a fixed kernel on the known "
                f"features, the kernel's own column over the path's time is {e['same_kernel_fixed_over_model']:.4f} "
                "(same kernel, same buffers)."]
        four = summarize_evaluation(path, families=("uniform", "banded", "poisson", "zipf"))
        if four and four["matrices"] != e["matrices"]:
            fb = names[four["best_fixed_kernel"]]
            out += ["", f"On the four families of BASELINE config 5 alone (uniform, banded, Poisson, Zipf; "
                    f"{four['matrices']} matrices, best fixed kernel {fb}): classifier selection "
                    f"{four['aggregate_speedup_vs_best_fixed']['classifier_selection']:.3f}x in total, "
                    f"{four['per_matrix_geomean_vs_best_fixed']['classifier_selection']:.3f}x per matrix; always gather "
                    f"{four['aggregate_speedup_vs_best_fixed']['always_gather']:.3f}x / "
                    f"{four['per_matrix_geomean_vs_best_fixed']['always_gather']:.3f}x."]
        c = summarize_evaluation(path, suffix="_cold")
        if c:
            cb = names[c["best_fixed_kernel"]]
            with open(path) as fh:
                n_cold = sum(int(r["cold_sets"]) > 1 for r in csv.DictReader(fh))
            out += ["", f"Cold (the {n_cold} matrices of at most 256 MiB timed on rotating copies of A, x, y -- up to "
                    f"{COLD_MAX_SETS}, more than 320 MiB in total where that many suffice --, the larger ones as above): "
                    f"best fixed kernel {cb} {c['t_fixed_us'][c['best_fixed_kernel']]:.0f} us, oracle {c['t_oracle_us']:.0f} us, "
                    f"always gather {c['t_always_gather_us']:.0f} us "
                    f"({c['aggregate_speedup_vs_best_fixed']['always_gather']:.3f}x in total, "
                    f"{c['per_matrix_geomean_vs_best_fixed']['always_gather']:.3f}x per matrix), classifier selection "
                    f"{c['t_classifier_selection_us']:.0f} us "
                    f"({c['aggregate_speedup_vs_best_fixed']['classifier_selection']:.3f}x / "
                    f"{c['per_matrix_geomean_vs_best_fixed']['classifier_selection']:.3f}x; "
                    f"{c['time_lost_vs_oracle']['classifier_selection']:.3f} of the oracle)."]
        # by family: where the classifier-selection path gains on the best fixed kernel and where it loses
        with open(path) as fh:
            rr = list(csv.DictReader(fh))
        Tk = np.array([[float(r[f"t_k{k}_us"]) for k in range(ND)] for r in rr])
        tm = np.array([float(r["t_model_us"]) + float(r.get("t_model_host_us") or 0.0) for r in rr])
        fam = np.array([r["family"] for r in rr])
        b = e["best_fixed_kernel"]
        out += ["", f"| family | matrices | {best} total us | classifier selection total us | oracle total us | "
                f"per-matrix geomean vs {best} | per-matrix geomean above oracle |", "|---|---|---|---|---|---|---|"]
        for f in list(dict.fromkeys(fam)):
            s_ = fam == f
            out.append(f"| {f} | {int(s_.sum())} | {Tk[s_, b].sum():.0f} | {tm[s_].sum():.0f} | {Tk[s_].min(axis=1).sum():.0f} | "
                       f"{np.exp(np.mean(np.log(Tk[s_, b] / tm[s_]))):.3f} | "
                       f"{np.exp(np.mean(np.log(tm[s_] / Tk[s_].min(axis=1)))):.3f} |")
        return out

    if eval_csv and os.path.exists(eval_csv):
        L += evaluation_section(eval_csv, "Held-out evaluation, every path re-measured end to end on the GPU timeline",
                                "the held-out matrices")
    if fresh_csv and os.path.exists(fresh_csv):
        with open(fresh_csv) as fh:
            ms = [int(r["m"]) for r in csv.DictReader(fh)]
        L += evaluation_section(fresh_csv, f"The same models on sweep numbers {min(ms)} to {max(ms)}, which no sweep or fit "
                                "has seen, re-measured end to end", "these matrices")
        L += ["", f"    python -m paper_2403_17017_amd.training evaluate --csv sweep.csv --model "
              f"paper_2403_17017_amd/selector_model.json --first {min(ms)} --count {len(ms)} --out eval_fresh.csv"]
    if "iterative" in m:
        it = m["iterative"]["report"]["test"]
        L += ["", "## Models for n products with one matrix (Sec. IV-E), held-out matrices, from sweep timings", "",
              "Cost of kernel k for n products: preprocessing(k) + n * run(k); the gathered path adds one "
              "feature-collection call.", "",
              "| n | best fixed kernel | classifier selection vs best fixed (aggregate) | per-matrix geomean | vs oracle | "
              "gathered on | preprocessing kernel chosen / truly best | amortisation called right |",
              "|---|---|---|---|---|---|---|---|"]
        for n, r in it.items():
            L.append(f"| {n} | {names[r['best_fixed_kernel']]} | {r['aggregate_speedup_vs_best_fixed']:.3f} | "
                     f"{r['per_matrix_geomean_vs_best_fixed']:.3f} | {r['time_lost_vs_oracle']:.3f} | "
                     f"{100 * r['gathered_fraction']:.0f} % | {100 * r['preprocessing_chosen_fraction']:.0f} % / "
                     f"{100 * r['preprocessing_best_fraction']:.0f} % | {100 * r['amortisation_accuracy']:.0f} % |")
    if iter_csv and os.path.exists(iter_csv):
        e = summarize_iterative_evaluation(iter_csv)
        with open(iter_csv) as fh:
            rr = list(csv.DictReader(fh))
        tp = lambda n, p: [float(r[f"t_plan_us_n{n}"]) for r in rr if int(r[f"path_n{n}"]) == p]
        L += ["", f"## The same models measured end to end ({e['matrices']} held-out matrices)", "",
              "    python -m paper_2403_17017_amd.training evaluate-iterative --model paper_2403_17017_amd/selector_model.json "
              "--out eval_iterative.csv", "",
              "Every kernel's preprocessing call and product timed again as in the sweep; the model's path = the "
              "seer_spmv_plan call as a user makes it through the Python binding (wall clock: selection, feature "
              "collection where asked for, preprocessing of the chosen kernel) + n * the product from the plan it "
              "returns (HIP graph replay).  The fixed kernels and the oracle are charged no call at all for kernels "
              "without preprocessing, so at n = 1 the path's own call decides the small matrices: it costs "
              f"{np.median(tp(1, 0)):.1f} us (median) on the known path, interpreter and ctypes included, and "
              f"{np.median(tp(19, 1)):.1f} us when it gathers.", "",
              "| n | best fixed kernel | classifier selection vs best fixed (aggregate) | per-matrix geomean | vs oracle | "
              "gathered on | preprocessing kernel chosen / truly best |",
              "|---|---|---|---|---|---|---|"]
        for n in ITER_EVAL_COUNTS:
            r = e[str(n)]
            L.append(f"| {n} | {names[r['best_fixed_kernel']]} | {r['aggregate_speedup_vs_best_fixed']:.3f} | "
                     f"{r['per_matrix_geomean_vs_best_fixed']:.3f} | {r['time_lost_vs_oracle']:.3f} | "
                     f"{100 * r['gathered_fraction']:.0f} % | {100 * r['preprocessing_chosen_fraction']:.0f} % / "
                     f"{100 * r['preprocessing_best_fraction']:.0f} % |")
    with open(out_md, "w") as fh:
        fh.write("\n".join(L) + "\n")
    return out_md


def _emit_node(tree, n, depth, lines):
    pad = "    " * depth
    if tree["feature"][n] < 0:
        lines.append(f"{pad}return {int(tree['klass'][n])};")
        return
    # hexadecimal floating constants are exact
    lines.append(f"{pad}if ((double)f[{int(tree['feature'][n])}] <= {float(tree['threshold'][n]).hex()}) {{")
    _emit_node(tree, tree["left"][n], depth + 1, lines)
    lines.append(f"{pad}}} else {{")
    _emit_node(tree, tree["right"][n], depth + 1, lines)
    lines.append(f"{pad}}}")


def export_header(model_json, out_h, prefix="seer_model"):
    """Writes the trained trees as a C header of nested if/else statements (the form the
    paper deploys its models in, Sec. III-D): one `static inline int <prefix>_<tree>(const
    float *f)` per tree, f being the 13-entry feature vector.  Readable, diffable, and
    equivalent to walking the node arrays."""
    with open(model_json) as fh:
        m = json.load(fh)
    names = m.get("feature_names", list(S.FEATURE_NAMES))
    lines = ["/* Generated by paper_2403_17017_amd.training export-header; do not edit.",
             f" * {m.get('note', '')}", " * Feature vector f[]: " + ", ".join(f"{i} {n}" for i, n in enumerate(names)),
             " * Return values: kernel ids 0 CSR,TM  1 CSR,WM  2 CSR,BM  3 CSR,MP  4 CSR,WO  5 CSR,A  6 ELL,TM  7 COO,WM  8 CSR,S;",
             " * the selector returns 0 = use the known model, 1 = gather features first. */",
             "#ifndef SEER_MODEL_GENERATED_H", "#define SEER_MODEL_GENERATED_H", ""]
    groups = [("", m)] + ([("_iterative", m["iterative"])] if "iterative" in m else [])
    for suffix, grp in groups:
        if suffix:
            lines += ["/* Models for several products with one matrix: f[12] is the iteration count. */", ""]
        for key in ("known", "gathered", "selector"):
            if key not in grp:
                continue
            lines.append(f"static inline int {prefix}{suffix}_{key}(const float *f)")
            lines.append("{")
            _emit_node(grp[key], 0, 1, lines)
            lines.append("}")
            lines.append("")
    # The gathered model of the single-product path is walked on the device, which needs the
    # node array rather than code: the same tree once more, as data, for users of the C ABI.
    g = m["gathered"]
    lines += ["#ifdef SEER_H   /* only where include/seer.h has been included before this file */",
              f"static const seer_node {prefix}_gathered_nodes[{len(g['feature'])}] = {{"]
    for i in range(len(g["feature"])):
        lines.append(f"    {{{int(g['feature'][i])}, {int(g['left'][i])}, {int(g['right'][i])}, {int(g['klass'][i])}, "
                     f"{float(g['threshold'][i]).hex()}}},")
    lines += ["};",
              f"static const seer_tree {prefix}_gathered_tree = {{{len(g['feature'])}, {len(names)}, {S.NUM_KERNELS}, "
              f"{prefix}_gathered_nodes}};",
              "#endif", "", "#endif"]
    with open(out_h, "w") as fh:
        fh.write("\n".join(lines) + "\n")
    return out_h


def _tree_from(d):
    return S.Tree(d["feature"], d["threshold"], d["left"], d["right"], d["klass"])


def load_model(path, iterative=False):
    """The single-product model, or with iterative=True the one for several products
    with one matrix (what seer_spmv_plan takes)."""
    with open(path) as fh:
        m = json.load(fh)
    grp = m["iterative"] if iterative else m
    sel = _tree_from(grp["selector"])
    sel.c.n_classes = 2
    return S.Model(_tree_from(grp["gathered"]), _tree_from(grp["known"]), sel), m


def load_tree(path):
    with open(path) as fh:
        t = json.load(fh)
    return S.Tree(t["feature"], t["threshold"], t["left"], t["right"], t["klass"]), t


def main(argv=None):
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    a = sub.add_parser("sweep")
    a.add_argument("--first", type=int, default=0)
    a.add_argument("--count", type=int, default=3000)
    a.add_argument("--out", default="sweep.csv")
    a.add_argument("--nnz-cap", type=int, default=200_000_000)
    a.add_argument("--max-rows-exp", type=float, default=7.0)
    a2 = sub.add_parser("sweep-slab", help="the CSR,S columns alone, for merging into an earlier sweep")
    a2.add_argument("--first", type=int, default=0)
    a2.add_argument("--count", type=int, default=3000)
    a2.add_argument("--out", default="sweep_slab.csv")
    a4 = sub.add_parser("sweep-cold", help="the cold columns alone (kernels without preprocessing on rotating copies)")
    a4.add_argument("--first", type=int, default=0)
    a4.add_argument("--count", type=int, default=3000)
    a4.add_argument("--out", default="sweep_cold.csv")
    a3 = sub.add_parser("merge")
    a3.add_argument("--csv", required=True)
    a3.add_argument("--extra", required=True)
    a3.add_argument("--out", required=True)
    b = sub.add_parser("fit")
    b.add_argument("--csv", required=True)
    b.add_argument("--out", default=os.path.join(os.path.dirname(__file__), "selector_model.json"))
    c = sub.add_parser("evaluate")
    c.add_argument("--csv", required=True)
    c.add_argument("--model", default=os.path.join(os.path.dirname(__file__), "selector_model.json"))
    c.add_argument("--out", default="eval.csv")
    c.add_argument("--first", type=int, default=None, help="with --count: evaluate on these sweep numbers instead "
                   "of the model's held-out ones (numbers beyond the fitted sweep are matrices no fit has seen)")
    c.add_argument("--count", type=int, default=0)
    ci = sub.add_parser("evaluate-iterative")
    ci.add_argument("--model", default=os.path.join(os.path.dirname(__file__), "selector_model.json"))
    ci.add_argument("--out", default="eval_iterative.csv")
    ci.add_argument("--first", type=int, default=None)
    ci.add_argument("--count", type=int, default=0)
    d = sub.add_parser("export-header")
    d.add_argument("--model", default=os.path.join(os.path.dirname(__file__), "selector_model.json"))
    d.add_argument("--out", default=os.path.join(os.path.dirname(__file__), "selector_model_generated.h"))
    e = sub.add_parser("report-md")
    e.add_argument("--csv", required=True)
    e.add_argument("--model", default=os.path.join(os.path.dirname(__file__), "selector_model.json"))
    e.add_argument("--eval", default=None)
    e.add_argument("--fresh-eval", default=None, help="evaluate --first/--count output on unseen sweep numbers")
    e.add_argument("--iterative-eval", default=None, help="evaluate-iterative output")
    e.add_argument("--out", required=True)
    args = ap.parse_args(argv)
    if args.cmd == "report-md":
        print(write_report_md(args.csv, args.model, args.eval, args.out, args.fresh_eval, args.iterative_eval))
        return
    if args.cmd == "export-header":
        print(export_header(args.model, args.out))
        return
    if args.cmd == "sweep-cold":
        run_cold_sweep(range(args.first, args.first + args.count), args.out)
    elif args.cmd == "sweep-slab":
        run_slab_sweep(range(args.first, args.first + args.count), args.out)
    elif args.cmd == "merge":
        print(merge_columns(args.csv, args.extra, args.out))
    elif args.cmd == "sweep":
        run_sweep(range(args.first, args.first + args.count), args.out, args.nnz_cap, args.max_rows_exp)
    elif args.cmd == "fit":
        m = fit_model(args.csv, args.out)
        print(json.dumps(m["report"], indent=1))
    elif args.cmd == "evaluate-iterative":
        fresh = None if args.first is None else list(range(args.first, args.first + args.count))
        print(json.dumps(evaluate_iterative(args.model, args.out, matrices=fresh), indent=1))
    else:
        fresh = None if args.first is None else list(range(args.first, args.first + args.count))
        print(json.dumps(evaluate_model(args.csv, args.model, args.out, matrices=fresh), indent=1))


if __name__ == "__main__":
    main()
