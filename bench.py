#!/usr/bin/env python3
"""Benchmark of the Seer SpMV hot path on one MI355X.

One step = one pass of the whole path over one matrix that is already resident in
HBM: gather the features of the matrix, walk the decision tree, run the SpMV schedule
it names -- seer_spmv_auto, which does all three on the device, enqueued back to
back.  The matrix is BASELINE config 2 (5-point Laplacian on a 1024 x 1024 grid).
Because that matrix (54 MB) fits the 256 MB last-level cache, the step rotates
through enough independent copies of (A, x, y) to exceed 1 GiB, so every launch
streams its operands from HBM.

Prints ONE JSON line.  value = model bytes per step / wall time per step, with
model bytes = 8 nnz + 4 (rows + 1) + 4 cols + 4 rows.  The `roofline` object prices
the selected SpMV kernel alone against the 8 TB/s HBM peak; `cpu_baseline` is the CPU
oracle on the same matrix; `extras` holds the same step through the three separate
calls (seer_features / seer_select / seer_spmv, host in the loop), every fixed
schedule cold and warm, and the selector measured on held-out sweep matrices.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
METRIC = "SpMV achieved HBM GB/s (% of peak) + selected-vs-best-single-kernel speedup"
COLD_BYTES = 1 << 30
CAL_WORDS = 1 << 26   # the calibration copy moves 256 MiB in and 256 MiB out
MODEL_PATH = os.path.join(ROOT, "paper_2403_17017_amd", "selector_model.json")


def make_workload(name: str):
    from workloads import csr_gen as G
    if name == "fixed16_4096":
        return G.fixed_degree()
    if name == "laplace5_1024":
        return G.laplacian_5pt(1024)
    if name == "zipf1.85_2M":
        return G.zipf_rows(s=1.85)
    if name == "zipf1.6_2M":
        return G.zipf_rows(s=1.6)
    if name == "empty30_poisson4_8M":
        return G.empty_poisson()
    if name == "laplace5_4096":
        return G.laplacian_5pt(4096)
    raise SystemExit(f"unknown workload {name}")


def load_model():
    """The shipped trees (known, gathered, classifier selection); a hand-written
    gathered tree only if the trained file is missing."""
    import paper_2403_17017_amd as S
    if os.path.exists(MODEL_PATH):
        from paper_2403_17017_amd.training import load_model as _load
        model, meta = _load(MODEL_PATH)
        return model, meta, meta.get("note", "trained")
    # var_len <= 50 ? CSR,BM : CSR,MP
    t = S.Tree([6, -1, -1], [50.0, 0, 0], [1, -1, -1], [2, -1, -1], [-1, 2, 3])
    return S.Model(t), {}, "hand-written default (no trained model file)"


def kernel_source_sha16():
    """Fingerprint of the device code (every file under csrc/): a profile summary taken from
    other sources is stale."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2403_17017_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".hiph", ".h")):
            with open(os.path.join(d, name), "rb") as fh:
                h.update(name.encode() + b"\0" + fh.read())
    return h.hexdigest()[:16]


def _read_summary(path):
    vals = {}
    with open(path) as fh:
        for ln in fh:
            if ":" in ln and not ln.startswith("#"):
                k, v = ln.split(":", 1)
                vals[k.strip()] = v.strip()
    return vals


def load_profile_summaries(workload, kernel):
    """What the committed rocprofv3 summaries say about the dominant kernel of this workload:
    HBM bytes per launch (two --pmc runs, FETCH_SIZE and WRITE_SIZE, calibrated against the
    plain copy kernel: counters cannot be read from inside a timed run) and the kernel-trace
    average duration.  Each summary names the kernel it was taken for and carries the
    fingerprint of the device sources it was taken from; a summary for another kernel counts
    as absent, one from other sources is reported as stale and its traffic figure withheld."""
    out = {"traffic": None, "traffic_file": None, "traffic_stale": None,
           "profile_avg_launch_us": None, "profile_file": None, "profile_stale": None}
    sha = kernel_source_sha16()
    tpath = os.path.join(ROOT, "profiles", f"traffic_{workload}.txt")
    if os.path.exists(tpath):
        v = _read_summary(tpath)
        if v.get("kernel") == kernel and "hbm_bytes_per_launch" in v:
            out["traffic_file"] = os.path.relpath(tpath, ROOT)
            out["traffic_stale"] = v.get("source_sha16") != sha
            if not out["traffic_stale"]:
                out["traffic"] = int(float(v["hbm_bytes_per_launch"]))
            else:
                out["traffic_of_stale_summary"] = int(float(v["hbm_bytes_per_launch"]))
    kpath = os.path.join(ROOT, "profiles", f"kernel_trace_{workload}.txt")
    if os.path.exists(kpath):
        v = _read_summary(kpath)
        if v.get("kernel") == kernel and "average_ns" in v:
            out["profile_file"] = os.path.relpath(kpath, ROOT)
            out["profile_avg_launch_us"] = round(float(v["average_ns"]) * 1e-3, 3)
            out["profile_stale"] = v.get("source_sha16") != sha
    return out


class Rotation:
    """n independent device copies of (A, x, y, workspace), carved out of ONE device allocation.

    One large allocation is mapped with large translation fragments; as n x 5 separate tensors the
    same copies made CSR,TM on the 54 MB Laplacian 3 to 4 % slower (11.4 against 11.0 us cold: a
    kernel that touches each page once per launch pays for every translation it misses)."""

    ALIGN = 4096

    def __init__(self, A, x, n):
        import torch

        import paper_2403_17017_amd as S
        up = lambda b: (b + self.ALIGN - 1) // self.ALIGN * self.ALIGN
        ws_bytes = max([S.spmv_auto_workspace_bytes(A.rows, A.nnz), S.features_workspace_bytes(A.rows)] +
                       [S.spmv_workspace_bytes(k, A.rows, A.nnz) for k in range(S.NUM_KERNELS)])
        sizes = [(A.rows + 1) * 4, max(A.nnz, 1) * 4, max(A.nnz, 1) * 4, max(A.cols, 1) * 4, max(A.rows, 1) * 4, max(ws_bytes, 256)]
        per = sum(up(b) for b in sizes)
        self.pool = torch.empty(per * n + self.ALIGN, dtype=torch.uint8, device="cuda:0")
        first = (-self.pool.data_ptr()) % self.ALIGN
        host = [torch.from_numpy(A.row_ptr), torch.from_numpy(A.col_idx), torch.from_numpy(A.values), torch.from_numpy(x)]
        self.sets = []
        for i in range(n):
            o, part = first + i * per, []
            for b in sizes:
                part.append(self.pool[o:o + b])
                o += up(b)
            rp, ci = part[0].view(torch.int32), part[1].view(torch.int32)[:A.nnz]
            va, xd = part[2].view(torch.float32)[:A.nnz], part[3].view(torch.float32)[:A.cols]
            for dst, src in zip((rp, ci, va, xd), host):
                dst.copy_(src)
            host = [rp, ci, va, xd]                                    # the later copies come from the first, on the device
            self.sets.append((S.DeviceCSR(A.rows, A.cols, rp, ci, va, A.nnz), xd, part[4].view(torch.float32), part[5]))
        self.n = n

    def __getitem__(self, i):
        return self.sets[i % self.n]


def time_spmv_back_to_back(kid, rot, reps, warmup):
    """Average time per launch, launches issued back to back (events around the batch)."""
    import torch

    import paper_2403_17017_amd as S
    for i in range(warmup):
        d, x, y, ws = rot[i]
        S.seer_spmv(kid, d, x, y, workspace=ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        d, x, y, ws = rot[warmup + i]
        S.seer_spmv(kid, d, x, y, workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps   # microseconds


def time_spmv_graph(kid, rot, reps, replays=3, prepared=False):
    """Average kernel time per launch with the launches replayed from one HIP graph,
    which takes the host's launch cost out of the measurement.  prepared: through
    seer_spmv_prepared from one plan per rotating copy (the kernels with preprocessing)."""
    import torch

    import paper_2403_17017_amd as S
    if prepared:
        plans = [S.seer_spmv_prepare(kid, rot[i][0]) for i in range(rot.n)]
        wss = [S.alloc_workspace(max(S.spmv_prepared_workspace_bytes(p_), 256)) for p_ in plans]

        def launch(i):
            d, x, y, _ = rot[i]
            S.seer_spmv_prepared(plans[i % rot.n], d, x, y, wss[i % rot.n])
    else:
        def launch(i):
            d, x, y, ws = rot[i]
            S.seer_spmv(kid, d, x, y, workspace=ws)
    for i in range(min(reps, rot.n)):
        launch(i)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(reps):
            launch(i)
    for _ in range(2):          # untimed: the first replays after other work run up to 2 % slower (clocks, caches)
        g.replay()
    torch.cuda.synchronize()
    total = 0.0
    for _ in range(replays):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        total += e0.elapsed_time(e1) * 1e3 / reps
    del g
    return total / replays


def stream_copy_ceiling(nbytes=1 << 31, reps=10):
    import torch

    import paper_2403_17017_amd as S
    a = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda:0").normal_()
    b = torch.empty_like(a)
    for _ in range(2):
        S.seer_stream_copy(b, a)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        S.seer_stream_copy(b, a)
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def stream_read_ceiling(nbytes=1 << 31, reps=10):
    """Rate of the library's read-only streaming kernel over a buffer far beyond the caches:
    the attainable rate of the access pattern an SpMV mostly is."""
    import torch

    import paper_2403_17017_amd as S
    a = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda:0").normal_()
    out = torch.zeros(64, dtype=torch.int32, device="cuda:0")
    for _ in range(2):
        S.seer_stream_sum(a, out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        S.seer_stream_sum(a, out)
    e1.record()
    torch.cuda.synchronize()
    return nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def random_gather_ceiling(nnz, cols, reps=10):
    """Rate of the library's bare gather kernel (streamed indices and values, no rows) with
    uniformly random indices into a vector of `cols` floats: what a product with random
    columns and this size of x can reach at most.  Returns gathers per second."""
    import torch

    import paper_2403_17017_amd as S
    n = max(4, min(int(nnz), 1 << 27) // 4 * 4)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(99)
    idx = torch.randint(0, max(int(cols), 1), (n,), generator=gen, device="cuda:0", dtype=torch.int32)
    val = torch.ones(n, dtype=torch.float32, device="cuda:0")
    x = torch.ones(max(int(cols), 1), dtype=torch.float32, device="cuda:0")
    out = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    for _ in range(3):
        S.seer_gather_sum(idx, val, x, out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        S.seer_gather_sum(idx, val, x, out)
    e1.record()
    torch.cuda.synchronize()
    return n * reps / (e0.elapsed_time(e1) * 1e-3)


def T_graph(enqueue):
    from paper_2403_17017_amd.training import time_graph_us
    return time_graph_us(enqueue, warmup=10, reps=20)


def selector_eval(model, meta, count):
    """Selected-vs-best-single-kernel on held-out matrices of the sweep population,
    every path timed on the GPU timeline (HIP graph replay, warm buffers)."""
    import torch

    import paper_2403_17017_amd as S
    from paper_2403_17017_amd import training as T
    from workloads.sweep_gen import build_on_device, sweep_spec
    tk, ta, tm = [], [], []
    for m in meta["test_matrices"][:count]:
        spec = sweep_spec(m)
        rp, ci, va, x = build_on_device(spec)
        dA = S.DeviceCSR(spec.rows, spec.rows, rp, ci, va, int(ci.numel()))
        ws = S.alloc_workspace(S.spmv_auto_workspace_bytes(dA.rows, dA.nnz))
        y = torch.empty(dA.rows, device="cuda:0")
        tk.append([T.time_kernel_us(k, dA, x, y, ws) for k in range(S.NUM_DIRECT_KERNELS)])
        ta.append(T.time_graph_us(lambda: S.seer_spmv_auto(dA, model.gathered, x, y, ws)))
        tm.append(T.time_graph_us(lambda: S.seer_spmv_model(dA, model, x, y, ws))
                  + S.seer_model_host_ns(model, dA.rows, dA.cols, dA.nnz) * 1e-3)   # + its host-side decision
        del rp, ci, va, x, dA, y, ws
    import numpy as np
    tk, ta, tm = np.array(tk), np.array(ta), np.array(tm)
    fixed = tk.sum(axis=0)
    best = int(np.argmin(fixed))
    geo = lambda a, b: float(np.exp(np.mean(np.log(a / b))))
    return {
        "protocol": "every path by one protocol (10 eager warm-up calls, 10 calls in one HIP graph, one untimed replay, "
                    "median of three timed replays), same buffers (warm); the classifier-selection path includes its "
                    "host-side decision (wall clock)",
        "matrices": len(tk), "best_fixed_kernel": S.kernel_name(best),
        "t_fixed_us": [round(float(v), 1) for v in fixed], "t_oracle_us": round(float(tk.min(axis=1).sum()), 1),
        "t_always_gather_us": round(float(ta.sum()), 1), "t_classifier_selection_us": round(float(tm.sum()), 1),
        "aggregate_speedup_vs_best_fixed": {"always_gather": round(float(fixed[best] / ta.sum()), 4),
                                            "classifier_selection": round(float(fixed[best] / tm.sum()), 4)},
        "per_matrix_geomean_vs_best_fixed": {"always_gather": round(geo(tk[:, best], ta), 4),
                                             "classifier_selection": round(geo(tk[:, best], tm), 4)},
    }


BASELINE_CONFIGS = (("fixed16_4096", "BASELINE config 1"), ("laplace5_1024", "BASELINE config 2"),
                    ("zipf1.6_2M", "BASELINE config 3 as stated (Zipf 1.6: 4.8e8 nonzeros)"),
                    ("zipf1.85_2M", "BASELINE config 3 at its stated size (Zipf 1.85: 4.7e7 nonzeros)"),
                    ("empty30_poisson4_8M", "BASELINE config 4"))
MAX_SETS = 2048


def config_row(name, what, tree, rot=None, per=None):
    """One BASELINE config under the cold protocol: every kernel without preprocessing
    (kernel time per launch, HIP graph replay on rotating copies), what seer_spmv_auto selects
    with the shipped tree, and the whole step."""
    import torch

    import paper_2403_17017_amd as S
    from workloads.csr_gen import dense_vector, model_bytes
    if rot is None:
        A = make_workload(name)
        x = dense_vector(A.cols, 12345)
        mb = model_bytes(A.rows, A.cols, A.nnz)
        rot = Rotation(A, x, min(MAX_SETS, max(1, math.ceil(COLD_BYTES / mb)) + 1))
        del A, x
    d0 = rot[0][0]
    mb = 8 * d0.nnz + 4 * (d0.rows + 1) + 4 * d0.cols + 4 * d0.rows
    # enough launches per replay that the replay's own fixed cost (about 10 us) stays under 1 % of it
    reps = 200 if mb < 100e6 else (20 if mb < 1e9 else 3)
    if per is None:      # (the bench's own workload hands over what its per-kernel table has just measured on these copies)
        per = {}
        for k in range(S.NUM_DIRECT_KERNELS):
            per[S.kernel_name(k)] = round(time_spmv_graph(k, rot, reps, replays=2 if mb > 1e9 else 3), 2)

    def enqueue_steps():
        for i in range(reps):
            d, xd, y, ws = rot[i]
            S.seer_spmv_auto(d, tree, xd, y, ws)
    from paper_2403_17017_amd.training import time_graph_us
    step = time_graph_us(enqueue_steps, warmup=1, reps=1) / reps
    _, kid = S.seer_spmv_auto_result(rot[0][3])
    sel = S.kernel_name(kid)
    best = min(per, key=per.get)
    gbps = lambda us: round(mb / (us * 1e-6) / 1e9, 1)
    return {
        "workload": name, "what": what, "rows": d0.rows, "cols": d0.cols, "nnz": d0.nnz, "model_bytes": mb,
        "cold_copies": rot.n, "per_kernel_cold_us": per,
        "selected_kernel": sel, "selected_cold_us": per[sel], "selected_gbps": gbps(per[sel]),
        "selected_frac_of_hbm_peak": round(gbps(per[sel]) / HBM_PEAK_GBPS, 4),
        "best_fixed_kernel": best, "best_fixed_cold_us": per[best], "best_fixed_gbps": gbps(per[best]),
        "best_fixed_frac_of_hbm_peak": round(gbps(per[best]) / HBM_PEAK_GBPS, 4),
        "step_us_gpu_timeline": round(step, 2), "step_gbps": gbps(step),
        "meets_60pct_of_hbm_peak": bool(gbps(per[best]) >= 0.6 * HBM_PEAK_GBPS),
    }


def cpu_baseline(A, x, tree, budget_s=10.0):
    """The oracle's whole step (features, tree walk, SpMV) on the host, single thread."""
    from oracle import seer_oracle as O
    from workloads.csr_gen import model_bytes
    reps, t_feat, t_spmv = 0, 0.0, 0.0
    t_start = time.perf_counter()
    while True:
        t0 = time.perf_counter()
        f = O.features(A.rows, A.cols, A.row_ptr)
        O.select(f["f"], *tree.arrays)
        t1 = time.perf_counter()
        O.spmv(A.rows, A.row_ptr, A.col_idx, A.values, x, want_bound=False)
        t2 = time.perf_counter()
        t_feat += t1 - t0
        t_spmv += t2 - t1
        reps += 1
        if time.perf_counter() - t_start > budget_s or reps >= 100000:
            break
    mb = model_bytes(A.rows, A.cols, A.nnz)
    # the same row loop with the rows shared among all host threads, timed for about 3 s
    y_all, threads = O.spmv_all_cores(A.rows, A.row_ptr, A.col_idx, A.values, x)
    n_all, t_all = 0, time.perf_counter()
    while time.perf_counter() - t_all < 3.0:
        O.spmv_all_cores(A.rows, A.row_ptr, A.col_idx, A.values, x)
        n_all += 1
    t_all = (time.perf_counter() - t_all) / n_all
    return {
        "spmv_all_cores": {"value": round(mb / t_all / 1e9, 4), "unit": "GB/s", "cores": threads,
                           "kind": "the oracle's row loop, rows shared among the host threads (OpenMP static)",
                           "spmv_ms": round(t_all * 1e3, 3)},
        "value": round(mb * reps / (t_feat + t_spmv) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"{reps} whole steps (oracle features + tree walk + fp64 C row loop) on the full "
                  f"{A.name} matrix, {t_feat + t_spmv:.1f} s of CPU time",
        "spmv_only_gbps": round(mb * reps / t_spmv / 1e9, 4),
        "spmv_ms": round(t_spmv / reps * 1e3, 3), "features_select_ms": round(t_feat / reps * 1e3, 3),
        "host_cpus": os.cpu_count(),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="laplace5_1024")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the per-kernel table and copy ceiling")
    ap.add_argument("--roofline-kernel", type=int, default=-1,
                    help="price this kernel id in `roofline` instead of the one the step selects (a kernel with "
                         "preprocessing is timed from prepared plans); for profiling a particular schedule")
    ap.add_argument("--size-scan", action="store_true",
                    help="extras.tm_size_scan: CSR,TM on 5-point Laplacians from 54 MB to 872 MB (adds about 10 s)")
    ap.add_argument("--no-configs", dest="configs", action="store_false",
                    help="skip the table of every BASELINE config in extras")
    ap.add_argument("--selector-matrices", type=int, default=60,
                    help="held-out sweep matrices for the selector figures in extras (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on exactly one GPU (--gpus 1); sharding over several GPUs is "
                         "not built")

    import torch

    import paper_2403_17017_amd as S
    from workloads.csr_gen import dense_vector, model_bytes

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    S.lib()   # fail now if the HIP library is missing
    A = make_workload(args.workload)
    x = dense_vector(A.cols, 12345)
    mb = model_bytes(A.rows, A.cols, A.nnz)
    n_sets = max(1, math.ceil(COLD_BYTES / mb)) + 1
    rot = Rotation(A, x, n_sets)
    model, model_meta, tree_note = load_model()
    tree = model.gathered

    def step(i):
        d, xd, y, ws = rot[i]
        S.seer_spmv_auto(d, tree, xd, y, ws)

    def three_call_step(i):
        d, xd, y, ws = rot[i]
        f = S.seer_features(d, workspace=ws)
        k = S.seer_select(f, tree)
        S.seer_spmv(k, d, xd, y, workspace=ws)
        return k

    # one plain copy of known size first: the calibration dispatch for byte counters
    cal_src = torch.empty(CAL_WORDS, dtype=torch.float32, device="cuda:0").normal_()
    cal_dst = torch.empty_like(cal_src)
    S.seer_stream_copy(cal_dst, cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    # W warm-up steps, then the K steps: enqueued once under HIP graph capture (the step has no
    # host-side dependency on device data, so it is capturable) and replayed -- one untimed
    # replay, then the timed one between two synchronizations.  Enqueued eagerly instead, the
    # four launches of a step cost the host about as long as the GPU needs for them, and the
    # figure would be the interpreter's (kept as extras.eager_ms_per_step).
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    eager_ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(args.steps):
            step(args.warmup + i)
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    graph.replay()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    del graph
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = mb / (ms_per_step * 1e-3) / 1e9
    f_dev, kid = S.seer_spmv_auto_result(rot[args.warmup + args.steps - 1][3])

    # Duration of the dominant kernel (the selected SpMV schedule): the same number of
    # launches on the same rotating copies, replayed from one HIP graph between two HIP
    # events, so that the figure is kernel time, free of launch gaps.
    rk = kid if args.roofline_kernel < 0 else args.roofline_kernel
    spmv_avg_us = time_spmv_graph(rk, rot, args.steps, replays=5, prepared=rk not in S.ONE_CALL_KERNELS or
                                  (rk >= S.NUM_DIRECT_KERNELS and args.roofline_kernel >= 0))
    achieved = mb / (spmv_avg_us * 1e-6) / 1e9
    prof = load_profile_summaries(args.workload + ("" if args.roofline_kernel < 0 else f"_k{rk}"), S.kernel_name(rk))
    out = {
        "metric": METRIC, "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{A.name}: {A.rows}x{A.cols} CSR, nnz={A.nnz}, fp32 values, int32 indices"
                               + (" (BASELINE config 2)" if args.workload == "laplace5_1024" else ""),
                   "step": "seer_spmv_auto = feature reduction + tree walk on the device + selected SpMV, "
                           "the K steps captured in one HIP graph and replayed",
                   "model_bytes_per_step": mb, "cache_protocol": f"cold: rotates {n_sets} copies of (A,x,y), "
                   f"{n_sets * mb / 2**30:.2f} GiB", "selected_kernel": S.kernel_name(kid), "tree": tree_note},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": prof["traffic"],
                     "kernel": S.kernel_name(rk), "avg_launch_us": round(spmv_avg_us, 3),
                     "meets_60pct_of_hbm_peak": bool(achieved >= 0.6 * HBM_PEAK_GBPS),
                     "profiles": {k: v for k, v in prof.items() if k != "traffic"},
                     "how": f"{args.steps} launches of the selected kernel on the rotating cold copies, "
                            "replayed from one HIP graph: mean of five replays, each bracketed by HIP events",
                     "algorithmic_bytes_per_launch": mb},
    }

    if not args.no_extras:
        extras = {"eager_ms_per_step": round(eager_ms_per_step, 5), "per_kernel_cold_us": {}, "per_kernel_warm_us": {}}
        warm = Rotation(A, x, 1)
        # launches per replay, as in config_row: the replay's fixed cost must stay small beside them
        table_reps = 200 if mb < 100e6 else (20 if mb < 1e9 else 3)
        for k in S.ONE_CALL_KERNELS:
            c = time_spmv_graph(k, rot, table_reps)
            w = time_spmv_graph(k, warm, table_reps)
            extras["per_kernel_cold_us"][S.kernel_name(k)] = round(c, 2)
            extras["per_kernel_warm_us"][S.kernel_name(k)] = round(w, 2)
        best = min(extras["per_kernel_cold_us"].values())
        # the kernels with preprocessing, from a prepared plan (one plan per rotating copy)
        extras["prepared_cold_us"], extras["prepared_warm_us"], extras["prepare_call_us"] = {}, {}, {}
        max_len = int(S.seer_features(warm[0][0]).max_len)
        for k in (S.CSR_A, S.ELL_TM, S.COO_WM, S.CSR_S):
            if k == S.ELL_TM and S.ell_plan_bytes(A.rows, max_len) == 0:
                continue                                   # padded arrays beyond 2^31 words: not applicable
            if k == S.CSR_S and S.slab_plan_bytes(A.rows, A.cols, A.nnz) == 0:
                continue                                   # x is a single slab: not applicable
            for R, key in ((rot, "prepared_cold_us"), (warm, "prepared_warm_us")):
                plans = [S.seer_spmv_prepare(k, R[i][0]) for i in range(R.n)]
                # (a plan's products may need more scratch than the one-call kernels: CSR,S keeps its partials there)
                wss = [S.alloc_workspace(max(S.spmv_prepared_workspace_bytes(p_), 256)) for p_ in plans]
                reps = table_reps

                def enqueue_all():
                    for i in range(reps):
                        d, xd, y, _ = R[i]
                        S.seer_spmv_prepared(plans[i % R.n], d, xd, y, wss[i % R.n])
                from paper_2403_17017_amd.training import time_graph_us
                extras[key][S.kernel_name(k)] = round(time_graph_us(enqueue_all, warmup=1, reps=1) / reps, 2)
                del plans, wss
            d = warm[0][0]
            pm = S.alloc_workspace(max(S.plan_bytes(k, A.rows, A.nnz), S.features_workspace_bytes(A.rows),
                                       S.ell_plan_bytes(A.rows, max_len) if k == S.ELL_TM else 0,
                                       S.slab_plan_bytes(A.rows, A.cols, A.nnz) if k == S.CSR_S else 0))
            S.seer_spmv_prepare(k, d, pm)
            t0 = time.perf_counter()
            for _ in range(10):
                S.seer_spmv_prepare(k, d, pm)
            extras["prepare_call_us"][S.kernel_name(k)] = round((time.perf_counter() - t0) / 10 * 1e6, 1)
            del pm
        extras["best_fixed_kernel_cold_gbps"] = round(mb / (best * 1e-6) / 1e9, 1)
        # the same step with the host in the loop: three calls, one wait
        for i in range(10):
            three_call_step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(100):
            three_call_step(i)
        torch.cuda.synchronize()
        extras["three_call_step_us"] = round((time.perf_counter() - t0) / 100 * 1e6, 2)
        t0 = time.perf_counter()
        for i in range(50):
            d, xd, y, ws = rot[i]
            S.seer_features(d, workspace=ws)
        extras["features_call_us"] = round((time.perf_counter() - t0) / 50 * 1e6, 2)
        # independent steps alternating between two streams (default priority): the short
        # launches of one step run under the product of the other.  Not the headline: that
        # one is one stream, one step after the other.
        lanes = [torch.cuda.Stream(), torch.cuda.Stream()]
        torch.cuda.synchronize()
        for rep in range(2):                                  # first round warms the streams
            t0 = time.perf_counter()
            for i in range(args.steps):
                d, xd, y, ws = rot[i]
                S.seer_spmv_auto(d, tree, xd, y, ws, stream=lanes[i & 1])
            torch.cuda.synchronize()
            extras["two_streams_us_per_step"] = round((time.perf_counter() - t0) / args.steps * 1e6, 2)
        # the classifier-selection path on this matrix (may skip gathering)
        d, xd, y, ws = rot[0]
        path, k_known = S.seer_spmv_model(d, model, xd, y, ws)
        extras["classifier_selection_on_this_matrix"] = {
            "path": "gathered" if path == 1 else "known",
            "kernel": S.kernel_name(S.seer_spmv_auto_result(ws)[1] if path == 1 else k_known)}
        # several products with one matrix (warm: a solver keeps using the same buffers):
        # selection with the iteration count + preprocessing of the chosen kernel + n products,
        # wall clock, against n products with the best kernel that needs no preprocessing
        if "iterative" in model_meta:
            from paper_2403_17017_amd.training import load_model as _load
            it_model, _ = _load(MODEL_PATH, iterative=True)
            d, xd, y, ws = warm[0]
            best_direct = min(extras["per_kernel_warm_us"][S.kernel_name(k)] for k in range(S.NUM_DIRECT_KERNELS))
            extras["iterative"] = {}
            # buffers a solver would allocate once: plan memory with room for the padded (ELL) form
            # of up to 1.5 x the CSR entries, the feature workspace, the products' workspace
            plan_mem = S.alloc_workspace(max(S.plan_bytes(S.CSR_A, d.rows, d.nnz), S.plan_bytes(S.COO_WM, d.rows, d.nnz),
                                             12 * d.nnz + (1 << 20), S.slab_plan_bytes(d.rows, d.cols, d.nnz)))
            fws = S.alloc_workspace(S.features_workspace_bytes(d.rows))
            # products' scratch: the most any plan for this matrix can ask for (CSR,S: its partials and carries)
            pws = S.alloc_workspace(max(S.spmv_workspace_bytes(k, d.rows, d.nnz) for k in range(S.NUM_KERNELS)) + 256
                                    + 4 * d.rows * (-(-d.cols >> 19)) + 8 * (d.nnz // 2048 + 64))
            for n_it in (1, 19, 100):
                wplan, _ = S.seer_spmv_plan(d, it_model, n_it, plan_mem, fws)   # warm the path once, the kernel's first launch included
                S.seer_spmv_prepared(wplan, d, xd, y, pws)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                plan, path = S.seer_spmv_plan(d, it_model, n_it, plan_mem, fws)
                for _ in range(n_it):
                    S.seer_spmv_prepared(plan, d, xd, y, pws)
                torch.cuda.synchronize()
                total = (time.perf_counter() - t0) * 1e6
                g = T_graph(lambda: S.seer_spmv_prepared(plan, d, xd, y, pws))
                extras["iterative"][str(n_it)] = {
                    "kernel": S.kernel_name(plan.kernel_id), "path": "gathered" if path == 1 else "known",
                    "wall_us_select_prepare_and_n_products": round(total, 1),
                    "product_us_on_gpu_timeline": round(g, 2),
                    "n_products_best_direct_kernel_us": round(n_it * best_direct, 1)}
        del warm
        extras["stream_copy_ceiling_gbps"] = round(stream_copy_ceiling(), 1)
        extras["read_ceiling_gbps"] = round(stream_read_ceiling(), 1)
        # warm, like the ceiling probe (which re-reads one set of buffers)
        extras["gathers"] = {
            "x_mb": round(A.cols * 4 / 1e6, 2),
            "random_gather_ceiling_per_s": round(random_gather_ceiling(A.nnz, A.cols), -6),
            "selected_kernel_per_s": round(A.nnz / (extras["per_kernel_warm_us"][S.kernel_name(kid)] * 1e-6), -6)}
        if model_meta.get("test_matrices") and args.selector_matrices > 0:
            extras["selector_on_held_out_matrices"] = selector_eval(model, model_meta, args.selector_matrices)
        if args.configs:
            # every BASELINE config under the same cold protocol (this workload's copies are reused)
            extras["configs"] = []
            for name, what in BASELINE_CONFIGS:
                if name == args.workload:
                    own = {S.kernel_name(k): extras["per_kernel_cold_us"][S.kernel_name(k)] for k in range(S.NUM_DIRECT_KERNELS)}
                    extras["configs"].append(config_row(name, what, tree, rot, own))
                    continue
                torch.cuda.empty_cache()
                extras["configs"].append(config_row(name, what, tree))
        if args.size_scan:
            # CSR,TM on 5-point Laplacians of growing size, same cold protocol: where a matrix
            # stops being one generation of workgroups and the kernel reaches its streaming rate
            from workloads import csr_gen as G
            extras["tm_size_scan"] = []
            for n in (1024, 1200, 1350, 1500, 1800, 2048, 2500, 3000, 3500, 4096):
                torch.cuda.empty_cache()
                L = G.laplacian_5pt(n)
                lb = model_bytes(L.rows, L.cols, L.nnz)
                lrot = Rotation(L, dense_vector(L.cols, 1), max(1, math.ceil(COLD_BYTES / lb)) + 1)
                t = time_spmv_graph(S.CSR_TM, lrot, 200 if lb < 100e6 else (60 if lb < 400e6 else 20))
                extras["tm_size_scan"].append({"grid": n, "model_bytes": lb, "cold_us": round(t, 2),
                                               "frac_of_hbm_peak": round(lb / (t * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)})
                del lrot, L
        out["extras"] = extras

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(A, x, tree)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
