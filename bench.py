#!/usr/bin/env python3
"""Benchmark of the tuned SpMV path on one MI355X.

One "step" is what the paper's tuned-SpMV experiment runs per matrix (Section VII-E, Eq. 2): extract the
features on the GPU, pick the format (decision tree / forest when a model file is present, otherwise the
run-first choice made before the timed region), then REPS = 1000 SpMVs in that format.  The headline value is
2 * nnz * REPS / t_step.  The one-off rows of the path (conversions, run-first tuning) and the SpMV rate of every
format are measured in the same run and printed in the same JSON line.

Workload: the 3-D 27-point stencil on a 128^3 grid in fp64 (synthetic, seeded), with
all inputs resident in HBM before the timed region starts.
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

HBM_PEAK_GBS = 8000.0
# HBM bytes per SpMV launch from the committed rocprofv3 counter runs (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, the scale
# factors a plain 1 GiB copy gives; see profiles/spmv_all_formats_stencil27_128_f64.md).  Keyed by (config, dtype, format).
MEASURED_TRAFFIC = {
    (2, "f64", "DIA"): 488.4e6, (2, "f64", "HDC"): 497.4e6, (2, "f64", "CSR"): 765.5e6, (2, "f64", "ELL"): 710.2e6,
    (2, "f64", "COO"): 959.4e6 + 9.1e6,
    # profiles/spmv_all_formats_banded_scatter_f64.md: the 1.17 M scattered entries gather one 128-byte line of x each
    (4, "f64", "HDC"): 535.3e6, (4, "f64", "CSR"): 736.2e6, (4, "f64", "ELL"): 784.5e6, (4, "f64", "HYB"): 684.9e6,
    (4, "f64", "COO"): 835.6e6 + 5.9e6,
    # profiles/spmv_all_formats_banded_scatter_f32.md
    (4, "f32", "HDC"): 331.4e6, (4, "f32", "HYB"): 482.6e6, (4, "f32", "CSR"): 502.8e6, (4, "f32", "ELL"): 565.9e6,
    (4, "f32", "COO"): 640.4e6 + 5.8e6,
    # profiles/spmv_all_formats_lognormal_f64.md: 16.8 M random gathers of x miss L2; bytes counted at the L2 boundary
    (3, "f64", "CSR"): 1333.9e6, (3, "f64", "HYB"): 659.5e6 + 722.1e6, (3, "f64", "COO"): 1524.7e6 + 8.4e6,
}
REPS = 1000
LLC_BYTES = 256 << 20     # last-level (Infinity) cache of the MI355X
MODEL_PATH = os.path.join(ROOT, "paper_2303_05098_amd", "models", "mi355x_forest.bin")


def algorithmic_bytes(fmt, v, sv):
    """Bytes one SpMV has to move in each format (x read once, y written once; padding slots count)."""
    m, n, nnz = v.m, v.n, v.nnz
    xy = n * sv + m * sv
    if fmt == 0:
        return nnz * (sv + 8) + xy
    if fmt == 1:
        return nnz * (sv + 4) + (m + 1) * 4 + xy
    if fmt == 2:
        return v.nd * m * sv + v.nd * 4 + xy
    if fmt == 3:
        return v.k * m * (sv + 4) + xy
    if fmt == 4:
        return v.k * m * (sv + 4) + v.nnz_coo * (sv + 8) + xy
    return v.nd * m * sv + v.nd * 4 + v.nnz_csr * (sv + 4) + (m + 1) * 4 + xy


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=2, help="2 = 27-point stencil 128^3 (default), 4 = banded+scatter, 3 = lognormal")
    ap.add_argument("--dtype", default="f64", choices=["f64", "f32"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copies", type=int, default=0,
                    help="device copies of each format the SpMV launches rotate over; 0 = as many as it takes for their "
                         "bytes to exceed twice the 256 MB last-level cache (at most 4), so that the streams come from HBM")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain 1 GiB -> 1 GiB device copy five times, as the known-size reference for HBM byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this library has no multi-GPU path; run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2303_05098_amd import mo, synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    np_dtype = np.float64 if args.dtype == "f64" else np.float32
    sv = 8 if args.dtype == "f64" else 4
    names = {1: "2-D 5-point Laplacian 64x64", 2: "3-D 27-point stencil 128^3", 3: "lognormal rows n=1048576",
             4: "banded+scatter n=4194304"}
    m, n, rp, ci, v = synth.config(args.config)
    nnz = int(rp[-1])
    x_host = synth.make_x(n, synth.BASE_SEED + args.config).astype(np_dtype)
    a = mo.Csr(m, n, rp, ci, np.asarray(v, dtype=np_dtype))
    x = torch.as_tensor(x_host).cuda()
    y = torch.empty(m, dtype=x.dtype, device="cuda")
    stream = torch.cuda.current_stream()
    ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731  (events on the stream the kernels are launched on)

    if args.calibrate:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    # ---- one-off rows of the path: features, conversions, per-format SpMV rate ------------------------------------
    t0 = time.perf_counter()
    feats, ints = mo.mo_features(a)
    torch.cuda.synchronize()
    t_fe_first = (time.perf_counter() - t0) * 1e3
    fe = []
    for _ in range(5):
        t0 = time.perf_counter()
        feats, ints = mo.mo_features(a)
        fe.append((time.perf_counter() - t0) * 1e3)
    t_fe = min(fe)

    handles, per_format, convert_ms = {}, {}, {}
    for fmt in range(6):
        t0 = time.perf_counter()
        try:
            h = mo.mo_convert(a, fmt)
        except mo.MoError as e:
            if e.status != mo.MO_E_FILL:
                raise
            per_format[mo.FORMAT_NAMES[fmt]] = None
            continue
        torch.cuda.synchronize()
        t_cold = (time.perf_counter() - t0) * 1e3
        # again with the allocator warm (the first repeat still has to get fresh blocks from the device, because `h`
        # holds the ones of the first call; after it is freed the caching allocator serves the same blocks again);
        # bytes = CSR arrays read + arrays of the format written (x and y taken out)
        t_warm = math.inf
        for rep in range(4):
            t0 = time.perf_counter()
            h2 = mo.mo_convert(a, fmt)
            torch.cuda.synchronize()
            if rep > 0:
                t_warm = min(t_warm, (time.perf_counter() - t0) * 1e3)
            h2.free()
        csr_bytes = nnz * (sv + 4) + (m + 1) * 4
        out_bytes = 0 if fmt == 1 else algorithmic_bytes(fmt, h.view(), sv) - (n + m) * sv
        convert_ms[mo.FORMAT_NAMES[fmt]] = {"first_call": round(t_cold, 3), "warm": round(t_warm, 3),
                                            "gbs": round((csr_bytes + out_bytes) / t_warm / 1e6, 1)}
        # A format whose arrays fit the last-level cache is timed over several copies in rotation (own device arrays
        # each, same contents), so that its value / index streams are read from HBM as they are at the other sizes.
        b = algorithmic_bytes(fmt, h.view(), sv)
        ncopies = args.copies if args.copies > 0 else (1 if b >= 1.25 * LLC_BYTES else min(4, math.ceil(2 * LLC_BYTES / b)))
        hs = [h] + [mo.mo_convert(a, fmt) for _ in range(ncopies - 1)]
        handles[fmt] = hs
        for i in range(10):
            mo.mo_spmv(hs[i % ncopies], x, y)
        best = math.inf
        for _ in range(5):
            e0, e1 = ev(), ev()
            e0.record(stream)
            for i in range(200):
                mo.mo_spmv(hs[i % ncopies], x, y)
            e1.record(stream)
            e1.synchronize()
            best = min(best, e0.elapsed_time(e1) / 200.0)
        per_format[mo.FORMAT_NAMES[fmt]] = {"us": round(best * 1e3, 2), "gflops": round(2.0 * nnz / best / 1e6, 1),
                                            "gbs": round(b / best / 1e6, 1), "frac_hbm": round(b / best / 1e6 / HBM_PEAK_GBS, 4),
                                            "alg_mbytes": round(b / 1e6, 1), "copies_in_rotation": ncopies}

    # ---- format choice ----------------------------------------------------------------------------------------------
    ms_vec = [per_format[nm]["us"] / 1e3 if per_format[nm] else float("nan") for nm in mo.FORMAT_NAMES]
    run_first = mo.mo_pick(ms_vec)
    model = mo.mo_model_load(MODEL_PATH) if os.path.exists(MODEL_PATH) else None
    if model is not None:
        t0 = time.perf_counter()
        for _ in range(1000):
            predicted = mo.mo_select(model, feats)
        t_pred_us = (time.perf_counter() - t0) * 1e3
        tuner = "random_forest" if model.info()[0] > 1 else "decision_tree"
        chosen = predicted if predicted in handles else run_first
    else:
        predicted, t_pred_us, tuner, chosen = None, None, "run_first", run_first
    hs = handles[chosen]
    h = hs[0]

    # ---- timed region: K steps of (features + select + REPS SpMVs in the chosen format) --------------------------
    def step(timed_events=None):
        f, _ = mo.mo_features(a)
        fmt = mo.mo_select(model, f) if model is not None else chosen
        hh = handles.get(fmt, hs)
        if timed_events is not None:
            timed_events[0].record(stream)
        for i in range(REPS):
            mo.mo_spmv(hh[i % len(hh)], x, y)
        if timed_events is not None:
            timed_events[1].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    kernel_events = [(ev(), ev()) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(kernel_events[k])
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t0
    ms_per_step = t_total * 1e3 / args.steps
    spmv_ms = sum(e0.elapsed_time(e1) for e0, e1 in kernel_events) / (args.steps * REPS)   # per launch
    value = 2.0 * nnz * REPS / (ms_per_step * 1e-3) / 1e9

    alg = algorithmic_bytes(chosen, h.view(), sv)
    achieved = alg / (spmv_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": {2: "k_dia_lds", 5: "k_dia_lds(HDC)", 1: "k_csr_tiled / k_csr_split", 3: "k_ell", 0: "k_coo_tile", 4: "k_ell+k_coo_tile"}[chosen],
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": MEASURED_TRAFFIC.get((args.config, args.dtype, mo.FORMAT_NAMES[chosen])), "algorithmic_bytes_per_launch": alg, "us_per_launch": round(spmv_ms * 1e3, 2)}

    # ---- run-first tuner (timed once; conversions included in its wall time) -------------------------------------------
    t0 = time.perf_counter()
    tune_best, tune_ms, _ = mo.mo_tune(a, warmups=5, reps=50)
    t_tune = (time.perf_counter() - t0) * 1e3

    # ---- the second operation: Y = A X with 8 right-hand sides, every format (not part of the timed step) ----------
    SPMM_K = 8
    xk = torch.as_tensor(np.ascontiguousarray(synth.uniform_pm1(synth.BASE_SEED + 40, 0, np.arange(n * SPMM_K)).reshape(n, SPMM_K),
                                              dtype=np_dtype)).cuda()
    yk = torch.empty((m, SPMM_K), dtype=xk.dtype, device="cuda")
    spmm = {}
    for fmt, hl in handles.items():
        hh = hl[0]
        for _ in range(3):
            mo.mo_spmm(hh, xk, yk)
        tb = math.inf
        for _ in range(3):
            e0, e1 = ev(), ev()
            e0.record(stream)
            for _ in range(20):
                mo.mo_spmm(hh, xk, yk)
            e1.record(stream)
            e1.synchronize()
            tb = min(tb, e0.elapsed_time(e1) / 20.0)
        bk = algorithmic_bytes(fmt, hh.view(), sv) + (SPMM_K - 1) * (n + m) * sv
        spmm[mo.FORMAT_NAMES[fmt]] = {"us": round(tb * 1e3, 1), "gflops": round(2.0 * nnz * SPMM_K / tb / 1e6, 1),
                                      "frac_hbm": round(bk / tb / 1e6 / HBM_PEAK_GBS, 4)}
    del xk, yk

    # ---- CPU baseline: the oracle, as it stands, on this host -------------------------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ref
        ti, tj, ta = ref.csr_to_triplets(rp, ci, np.asarray(v, dtype=np_dtype).astype(np.float64))
        xo = x_host.astype(np.float64)
        cores = len(os.sched_getaffinity(0))
        cores = min(cores, 16)
        t0 = time.perf_counter()
        y1, mag = ref.spmv(m, n, ti, tj, ta, xo)
        t_1 = time.perf_counter() - t0
        reps_mt, t_mt = 0, 0.0
        while t_mt < 8.0 and reps_mt < 50:
            t0 = time.perf_counter()
            ymt = ref.spmv_rowsorted_mt(m, ti, tj, ta, xo, cores)
            t_mt += time.perf_counter() - t0
            reps_mt += 1
        # the GPU result of the chosen format is checked against the oracle while we are here
        mo.mo_spmv(h, x, y)
        torch.cuda.synchronize()
        err, zeros_ok = ref.spmv_error(y.cpu().numpy(), y1, mag)
        cpu_model = "unknown"
        try:
            with open("/proc/cpuinfo") as fh:
                cpu_model = next((ln.split(":", 1)[1].strip() for ln in fh if ln.startswith("model name")), cpu_model)
        except OSError:
            pass
        cpu = {"value": round(2.0 * nnz / (t_mt / reps_mt) / 1e9, 3), "unit": "GFLOP/s", "cores": cores, "kind": "oracle",
               "sample": f"{reps_mt} full SpMVs of the workload matrix, long-double COO-triplet loop split over {cores} threads by row range",
               "single_thread_gflops": round(2.0 * nnz / t_1 / 1e9, 3), "cpu_model": cpu_model, "gpu_vs_oracle_max_rel_err": err, "zeros_ok": zeros_ok}

    csr_us = per_format["CSR"]["us"]
    best_us = per_format[mo.FORMAT_NAMES[chosen]]["us"]
    out = {
        "metric": "tuned SpMV GFLOP/s (features + format selection + 1000 SpMVs in the selected format, Eq. 2 form)",
        "value": round(value, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"{names[args.config]}, {args.dtype}, m={m}, nnz={nnz}", "spmv_reps_per_step": REPS, "tuner": tuner,
                   "matrix_copies_in_rotation": len(hs)},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "per_format": per_format,
        "selected_format": mo.FORMAT_NAMES[chosen],
        "run_first_format": mo.FORMAT_NAMES[run_first],
        "model_predicted_format": mo.FORMAT_NAMES[predicted] if predicted is not None else None,
        "speedup_vs_csr_spmv_only": round(csr_us / best_us, 3),
        "speedup_vs_csr_eq2": round(csr_us * 1e-3 * REPS / ms_per_step, 3),
        "t_fe_ms": round(t_fe, 3), "t_fe_first_call_ms": round(t_fe_first, 3),
        "features_gbs": round((nnz * 4 + (m + 1) * 4 + 2 * (m + n - 1) * 4) / t_fe / 1e6, 1),
        "t_pred_us": round(t_pred_us, 3) if t_pred_us is not None else None,
        "tuner_cost_in_csr_spmv": round((t_fe + (t_pred_us or 0.0) * 1e-3) / (csr_us * 1e-3), 1),
        "spmm_8_rhs_per_format": spmm,
        "convert_ms": convert_ms,
        "mo_tune": {"best": mo.FORMAT_NAMES[tune_best], "wall_ms": round(t_tune, 1),
                    "ms_per_rep": [None if math.isnan(t) else round(float(t), 5) for t in tune_ms]},
        "features": [float(f) for f in feats],
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
