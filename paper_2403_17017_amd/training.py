"""Training side of the selector (Sec. III-A and III-D of the Seer paper): benchmark
every SpMV schedule and the feature collection on a representative population, label
each matrix with its fastest schedule, fit a CART decision tree (scikit-learn, Gini,
depth-capped, 80/20 split, no hyper-parameter tuning) and store it as the flat node
array `seer_select` walks.

    python -m paper_2403_17017_amd.training sweep --count 1000 --out gpurun_out/sweep.csv
    python -m paper_2403_17017_amd.training fit --csv gpurun_out/sweep.csv \
           --out paper_2403_17017_amd/selector_tree.json

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
CSV_FIELDS = (["m", "family", "rows", "cols", "nnz"] + [f"f_{n}" for n in S.FEATURE_NAMES]
              + ["t_features_us"] + [f"t_k{k}_us" for k in range(S.NUM_KERNELS)] + ["max_disagreement"])


def time_kernel_us(kid, dA, x, y, ws, warmup=10, reps=10):
    import torch
    for _ in range(warmup):
        S.seer_spmv(kid, dA, x, y, workspace=ws)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(reps):
            S.seer_spmv(kid, dA, x, y, workspace=ws)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def time_features_us(dA, ws, warmup=3, reps=10):
    for _ in range(warmup):
        f = S.seer_features(dA, workspace=ws)
    t0 = time.perf_counter()
    for _ in range(reps):
        f = S.seer_features(dA, workspace=ws)
    return (time.perf_counter() - t0) / reps * 1e6, f


def measure_matrix(spec, device="cuda:0"):
    """One CSV row for sweep matrix `spec` (see workloads.sweep_gen)."""
    import torch

    from workloads.sweep_gen import build_on_device
    rp, ci, va, x = build_on_device(spec, device)
    dA = S.DeviceCSR(spec.rows, spec.rows, rp, ci, va, int(ci.numel()))
    ws = S.alloc_workspace(max(S.spmv_workspace_bytes(S.CSR_MP, dA.rows, dA.nnz),
                               S.features_workspace_bytes(dA.rows)), device)
    t_feat, f = time_features_us(dA, ws)
    row = {"m": spec.m, "family": spec.family, "rows": dA.rows, "cols": dA.cols, "nnz": dA.nnz,
           "t_features_us": round(t_feat, 3)}
    for n, v in zip(S.FEATURE_NAMES, f.vector()):
        row[f"f_{n}"] = repr(float(v))
    ys = []
    for k in range(S.NUM_KERNELS):
        y = torch.empty(dA.rows, device=device)
        row[f"t_k{k}_us"] = round(time_kernel_us(k, dA, x, y, ws), 3)
        ys.append(y)
    # the schedules must agree with each other (a sanity check, not the parity test)
    scale = float(ys[3].abs().max().item()) + 1e-30
    row["max_disagreement"] = float(max((ys[k] - ys[3]).abs().max().item() for k in range(3)) / scale)
    return row


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
                  f"t={[row[f't_k{k}_us'] for k in range(4)]} feat={row['t_features_us']} "
                  f"({time.time() - t_start:.0f}s)", file=log, flush=True)


def load_csv(path):
    with open(path) as fh:
        rows = list(csv.DictReader(fh))
    X = np.array([[float(r[f"f_{n}"]) for n in S.FEATURE_NAMES] for r in rows], dtype=np.float32)
    T = np.array([[float(r[f"t_k{k}_us"]) for k in range(S.NUM_KERNELS)] for r in rows])
    tf = np.array([float(r["t_features_us"]) for r in rows])
    return rows, X, T, tf


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


def fit_tree(csv_path, out_json, test_frac=0.2, seed=0):
    from sklearn.model_selection import train_test_split
    from sklearn.tree import DecisionTreeClassifier
    rows, X, T, tf = load_csv(csv_path)
    y = T.argmin(axis=1)            # ties -> lowest kernel id
    idx = np.arange(len(rows))
    tr, te = train_test_split(idx, test_size=test_frac, random_state=seed)
    clf = DecisionTreeClassifier(criterion="gini", max_depth=MAX_DEPTH, random_state=0).fit(X[tr], y[tr])
    tree = tree_to_arrays(clf)
    assert np.array_equal(predict_with_arrays(tree, X), clf.predict(X))
    report = {"train": selector_report(T[tr], tf[tr], clf.predict(X[tr])),
              "test": selector_report(T[te], tf[te], clf.predict(X[te])),
              "all": selector_report(T, tf, clf.predict(X))}
    tree.update({"note": f"CART gini max_depth={MAX_DEPTH}, {len(tr)} training matrices",
                 "feature_names": list(S.FEATURE_NAMES), "n_classes": S.NUM_KERNELS,
                 "label_counts": np.bincount(y, minlength=S.NUM_KERNELS).tolist(), "report": report})
    with open(out_json, "w") as fh:
        json.dump(tree, fh, indent=1)
    return tree


def load_tree(path):
    with open(path) as fh:
        t = json.load(fh)
    return S.Tree(t["feature"], t["threshold"], t["left"], t["right"], t["klass"]), t


def main(argv=None):
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    a = sub.add_parser("sweep")
    a.add_argument("--first", type=int, default=0)
    a.add_argument("--count", type=int, default=1000)
    a.add_argument("--out", default="gpurun_out/sweep.csv")
    a.add_argument("--nnz-cap", type=int, default=200_000_000)
    a.add_argument("--max-rows-exp", type=float, default=7.0)
    b = sub.add_parser("fit")
    b.add_argument("--csv", required=True)
    b.add_argument("--out", default=os.path.join(os.path.dirname(__file__), "selector_tree.json"))
    args = ap.parse_args(argv)
    if args.cmd == "sweep":
        run_sweep(range(args.first, args.first + args.count), args.out, args.nnz_cap, args.max_rows_exp)
    else:
        t = fit_tree(args.csv, args.out)
        print(json.dumps(t["report"], indent=1))


if __name__ == "__main__":
    main()
