"""CPU-only checks of the training-side harness: the sweep recipe is deterministic,
matrices it builds are valid CSR, and the CART fit recovers a planted rule."""
import csv

import numpy as np

import paper_2403_17017_amd as S
from paper_2403_17017_amd import training as T
from workloads import sweep_gen as W


def test_sweep_specs_are_deterministic_and_capped():
    fams = set()
    for m in range(40):
        a, b = W.sweep_spec(m, nnz_cap=2_000_000), W.sweep_spec(m, nnz_cap=2_000_000)
        assert a.family == b.family and a.rows == b.rows and np.array_equal(a.lens, b.lens)
        assert a.nnz <= 2_000_000 and a.lens.min() >= 0 and a.lens.max() <= a.rows
        fams.add(a.family)
    assert fams == set(W.FAMILIES)


def test_build_gives_valid_sorted_csr():
    for m in range(12):
        spec = W.sweep_spec(m, nnz_cap=300_000, max_rows_exp=4.5)
        rp, ci, va, x = W.build_on_device(spec, "cpu")
        rp, ci = rp.numpy().astype(np.int64), ci.numpy().astype(np.int64)
        assert rp[0] == 0 and rp[-1] == ci.size == va.numel() and x.numel() == spec.rows
        assert np.array_equal(np.diff(rp), spec.lens)
        if ci.size:
            assert ci.min() >= 0 and ci.max() < spec.rows
            row = np.repeat(np.arange(spec.rows), spec.lens)
            key = row * spec.rows + ci
            assert np.all(np.diff(key) >= 0)          # ascending inside rows
            if spec.family == "banded":
                assert np.all(np.abs(ci - row) <= spec.params["b"]) and np.all(np.diff(key) > 0)
        assert float(va.abs().max()) <= 1.0 if va.numel() else True


def test_fit_recovers_planted_rule(tmp_path):
    # kernel 2 is fastest iff var_len <= 40, else kernel 3; features cost 5 us
    rng = np.random.default_rng(0)
    p = tmp_path / "sweep.csv"
    with open(p, "w", newline="") as fh:
        w = csv.DictWriter(fh, fieldnames=T.CSV_FIELDS)
        w.writeheader()
        for m in range(300):
            f = np.exp(rng.normal(2, 2, S.NUM_FEATURES)).astype(np.float32)
            fast = 2 if f[6] <= 40 else 3
            t = [100.0, 90.0, 80.0, 70.0, 75.0, 16.0, float("inf"), 95.0, float("inf")]   # kernel 5 is a little faster per product ...
            t[fast] = 20.0
            row = {"m": m, "family": "x", "rows": int(f[0]) + 1, "cols": 1, "nnz": 1, "t_features_us": 5.0,
                   "max_disagreement": 0.0}
            row.update({f"f_{n}": repr(float(v)) for n, v in zip(S.FEATURE_NAMES, f)})
            row.update({f"t_k{k}_us": t[k] for k in range(S.NUM_KERNELS)})
            row["t_prep_k5_us"], row["t_single_k5_us"] = 60.0, 76.0   # ... but needs 60 us of preprocessing
            row["t_prep_k6_us"], row["t_single_k6_us"] = "inf", "inf"  # the ELL form applies to none of them
            row["t_prep_k7_us"], row["t_single_k7_us"] = 40.0, 135.0
            row["t_prep_k8_us"], row["t_single_k8_us"] = "inf", "inf"  # nor does the column-slabbed one
            row.update({f"t_rep_k{k}_us": t[k] for k in range(S.NUM_DIRECT_KERNELS)})
            row["t_auto_mp_us"] = t[3] + 4.0          # gathering on the device costs 4 us
            w.writerow(row)
    out = tmp_path / "model.json"
    model = T.fit_model(str(p), str(out))
    rep = model["report"]
    assert rep["test"]["accuracy"]["gathered"] == 1.0 and rep["train"]["accuracy"]["gathered"] == 1.0
    assert rep["test"]["accuracy"]["known"] < 0.9          # var_len is not a known feature
    assert abs(model["gather_overhead_us"]["intercept"] - 4.0) < 0.5
    assert rep["all"]["aggregate_speedup_vs_best_fixed"]["gathered"] > 1.2
    # gathering costs 4 us and saves 50-60 us whenever the known model is wrong: the selector gathers
    assert rep["all"]["gathered_fraction"] > 0.3
    assert rep["all"]["t_us"]["classifier_selection"] <= rep["all"]["t_us"]["known"]
    # the shipped format round-trips through the C ABI walker
    m, _ = T.load_model(str(out))
    from paper_2403_17017_amd import binding as B
    for v, want in ((10.0, 2), (400.0, 3)):
        f = B.seer_features_t()
        f.f[6] = v
        assert S.seer_select(f, m.gathered) == want
    assert all(f in (-1, 0, 1, 2, 3, 8) for f in model["known"]["feature"] + model["selector"]["feature"])
    assert max(model["gathered"]["klass"]) < S.NUM_DIRECT_KERNELS     # single products: no preprocessing
    # several products with one matrix: 60 + 16 n < 20 n from n = 16 on, so the preprocessing
    # kernel is the label for the grid's n >= 19 and never below
    it = model["iterative"]
    for n, r in it["report"]["test"].items():
        assert r["amortisation_accuracy_gathered"] == 1.0, n
        assert r["preprocessing_best_fraction"] == (1.0 if int(n) >= 16 else 0.0)
        assert r["accuracy"]["gathered"] == 1.0
    assert it["report"]["test"]["100"]["accuracy"]["known"] == 1.0     # the iteration count is known
    assert all(f in (-1, 0, 1, 2, 3, 8, 12) for f in it["known"]["feature"] + it["selector"]["feature"])
    mi, _ = T.load_model(str(out), iterative=True)
    f = B.seer_features_t()
    f.f[6], f.f[12] = 10.0, 3.0
    assert S.seer_select(f, mi.gathered) == 2
    f.f[12] = 50.0
    # (kernel 6 costs what kernel 5 costs wherever its format does not apply: either answer is right)
    assert S.seer_select(f, mi.gathered) in (5, 6, 8) and S.seer_select(f, mi.known) in (5, 6, 8)


def test_exported_header_is_equivalent_to_the_node_arrays(tmp_path):
    """The generated if/else header, compiled with gcc, answers like the oracle's tree
    walk on random vectors and on vectors that sit exactly on thresholds."""
    import ctypes
    import json
    import os
    import subprocess

    from oracle import seer_oracle as O
    model_path = os.path.join(os.path.dirname(T.__file__), "selector_model.json")
    hdr = T.export_header(model_path, str(tmp_path / "model.h"))
    src = tmp_path / "wrap.c"
    src.write_text('#include "model.h"\n'
                   "int known(const float *f) { return seer_model_known(f); }\n"
                   "int gathered(const float *f) { return seer_model_gathered(f); }\n"
                   "int selector(const float *f) { return seer_model_selector(f); }\n")
    so = tmp_path / "wrap.so"
    subprocess.check_call(["gcc", "-O1", "-shared", "-fPIC", "-I", str(tmp_path), "-o", str(so), str(src)])
    lib = ctypes.CDLL(str(so))
    m = json.load(open(model_path))
    rng = np.random.default_rng(3)
    for key in ("known", "gathered", "selector"):
        t = m[key]
        arrs = (t["feature"], t["threshold"], t["left"], t["right"], t["klass"])
        thr = [(f, th) for f, th in zip(t["feature"], t["threshold"]) if f >= 0]
        fn = getattr(lib, key)
        fn.argtypes = [ctypes.POINTER(ctypes.c_float)]
        for i in range(400):
            v = np.exp(rng.normal(4, 4, 12)).astype(np.float32)
            v[7] = rng.random()
            if thr and i % 2:
                f, th = thr[int(rng.integers(len(thr)))]
                v[f] = np.float32(th) if i % 4 == 1 else np.nextafter(np.float32(th), np.float32(np.inf))
            got = fn(v.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
            assert got == O.select(v, *arrs)
    assert "if ((double)f[" in open(hdr).read()


def test_committed_header_is_the_export_of_the_committed_model(tmp_path):
    """paper_2403_17017_amd/selector_model_generated.h is compiled into the library as its
    built-in model: it must be exactly what export-header writes for the committed
    selector_model.json, byte for byte."""
    import os
    here = os.path.dirname(T.__file__)
    fresh = T.export_header(os.path.join(here, "selector_model.json"), str(tmp_path / "fresh.h"))
    with open(fresh) as a, open(os.path.join(here, "selector_model_generated.h")) as b:
        assert a.read() == b.read(), "run `python -m paper_2403_17017_amd.training export-header` and rebuild"


def test_committed_model_is_the_fit_of_the_committed_sweep(tmp_path):
    """The shipped trees can be derived again from what the repository holds:
    selector_sweep.csv.gz (the timings of the 3000-matrix sweep, warm and cold columns,
    all nine kernels) fitted by `training fit` gives selector_model.json, value for value."""
    import json
    import os
    here = os.path.dirname(T.__file__)
    out = str(tmp_path / "refit.json")
    T.fit_model(os.path.join(here, "selector_sweep.csv.gz"), out)
    with open(out) as a, open(os.path.join(here, "selector_model.json")) as b:
        assert json.load(a) == json.load(b)
