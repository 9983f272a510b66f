"""Tuner sweep (benchmark configs[4]): the offline stage of the paper's pipeline (Section III-A) on synthetic
matrices.

    python -m paper_2303_05098_amd.sweep run --first 0 --count 64 --out gpurun_out/sweep_000.jsonl     (GPU)
    python -m paper_2303_05098_amd.sweep fit gpurun_out/sweep_*.jsonl --model paper_2303_05098_amd/models/mi355x_tree.bin

``run``: per matrix, features on the GPU (mo_features), then the run-first tuner (mo_tune, 1000 timed SpMVs per
feasible format as in Section VII-A); label = format with the smallest time.  ``fit``: stratified 5-fold
cross-validation of a depth-limited tree, accuracy and balanced accuracy (Section VII-C), geometric-mean speedup
over CSR of the true best and of the predicted format (SpMV only, and in the form of Eq. 2 with tuner time
included), then a tree fitted on all records is written as the model file mo_select loads.
"""
from __future__ import annotations

import argparse
import glob
import json
import math
import os
import sys
import time

import numpy as np

from . import fit as fitmod
from . import synth

FORMATS = ("COO", "CSR", "DIA", "ELL", "HYB", "HDC")


def run(first: int, count: int, out: str, reps: int, n_hi: float) -> None:
    import torch

    from . import mo

    with open(out, "a") as fh:
        for k in range(first, first + count):
            t0 = time.perf_counter()
            fam, m, n, rp, ci, v = synth.sweep_matrix(k, 1e3, n_hi)
            t_gen = time.perf_counter() - t0
            a = mo.Csr(m, n, rp, ci, v)
            mo.mo_features(a)                                   # first call pays allocator warm-up
            fe = []
            for _ in range(3):
                t0 = time.perf_counter()
                feats, ints = mo.mo_features(a)
                fe.append((time.perf_counter() - t0) * 1e3)
            best, ms, cv = mo.mo_tune(a, warmups=5, reps=reps)
            rec = dict(k=k, family=fam, m=m, n=n, nnz=int(rp[-1]), features=[float(f) for f in feats], t_fe_ms=min(fe),
                       ms_per_rep=[None if math.isnan(t) else float(t) for t in ms],
                       convert_ms=[None if math.isnan(t) else float(t) for t in cv], best=int(best), reps=reps)
            fh.write(json.dumps(rec) + "\n")
            fh.flush()
            print(f"[sweep] k={k} {fam} m={m} nnz={rec['nnz']} gen={t_gen:.1f}s best={FORMATS[best]} "
                  f"ms={[None if t is None else round(t, 4) for t in rec['ms_per_rep']]}", flush=True)
            del a
            torch.cuda.empty_cache()


def load(paths) -> list:
    recs = {}
    for p in paths:
        for line in open(p):
            line = line.strip()
            if line:
                r = json.loads(line)
                recs[r["k"]] = r
    return [recs[k] for k in sorted(recs)]


def geomean(v) -> float:
    v = np.asarray(v, dtype=np.float64)
    return float(np.exp(np.mean(np.log(v)))) if v.size else float("nan")


def analyse(recs, max_depth: int, min_samples_leaf: int, reps_eq2: int = 1000, t_pred_ms: float = 0.001) -> dict:
    X = np.array([r["features"] for r in recs], dtype=np.float64)
    ms = np.array([[np.nan if t is None else t for t in r["ms_per_rep"]] for r in recs], dtype=np.float64)
    y = np.array([r["best"] for r in recs], dtype=np.int64)
    cv = fitmod.cross_validate(X, y, 5, max_depth, min_samples_leaf)
    pred = cv["pred"]
    t_csr = ms[:, 1]
    t_best = ms[np.arange(len(recs)), y]
    # a predicted format that is infeasible for the matrix falls back to CSR, as a deployed tuner would
    t_pred = ms[np.arange(len(recs)), pred]
    t_pred = np.where(np.isnan(t_pred), t_csr, t_pred)
    t_fe = np.array([r["t_fe_ms"] for r in recs])
    eq2 = (t_csr * reps_eq2) / (t_fe + t_pred_ms + t_pred * reps_eq2)
    cost = (t_fe + t_pred_ms) / t_csr
    q = np.percentile(cost, [0, 25, 50, 75, 100])
    # SpMVs after which tuning has paid for itself, conversion included (the paper leaves conversion out of Eq. 2):
    # smallest n with t_fe + t_pred + t_conv + n * t_pred_fmt < n * t_csr; only where the predicted format is faster
    conv = np.array([[np.nan if t is None else t for t in r["convert_ms"]] for r in recs], dtype=np.float64)
    t_conv = conv[np.arange(len(recs)), pred]
    gain = t_csr - t_pred
    pays = (gain > 0) & (pred != 1) & ~np.isnan(t_conv)
    breakeven = np.ceil((t_fe + t_pred_ms + t_conv)[pays] / gain[pays])
    bq = np.percentile(breakeven, [25, 50, 75]) if breakeven.size else [float("nan")] * 3
    return dict(
        n=len(recs), class_histogram={FORMATS[c]: int((y == c).sum()) for c in range(6)},
        predicted_histogram={FORMATS[c]: int((pred == c).sum()) for c in range(6)},
        cv_accuracy=cv["accuracy"], cv_balanced_accuracy=cv["balanced_accuracy"], per_fold=cv["per_fold"],
        geomean_speedup_best_vs_csr=geomean(t_csr / t_best),
        geomean_speedup_predicted_vs_csr=geomean(t_csr / t_pred),
        geomean_speedup_eq2_predicted=geomean(eq2),
        max_speedup_best_vs_csr=float(np.max(t_csr / t_best)),
        mean_speedup_best_vs_csr_where_not_csr=float(np.mean((t_csr / t_best)[y != 1])) if (y != 1).any() else None,
        tuner_cost_in_csr_spmv=dict(mean=float(cost.mean()), std=float(cost.std()), min=float(q[0]), q1=float(q[1]),
                                    q2=float(q[2]), q3=float(q[3]), max=float(q[4])),
        breakeven_spmvs_incl_conversion=dict(n_matrices=int(pays.sum()), q1=float(bq[0]), q2=float(bq[1]), q3=float(bq[2])),
        max_depth=max_depth, min_samples_leaf=min_samples_leaf,
    ), X, y


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    r = sub.add_parser("run")
    r.add_argument("--first", type=int, default=0)
    r.add_argument("--count", type=int, default=256)
    r.add_argument("--out", required=True)
    r.add_argument("--reps", type=int, default=1000)
    r.add_argument("--n-hi", type=float, default=4e6)
    f = sub.add_parser("fit")
    f.add_argument("records", nargs="+")
    f.add_argument("--model", default=None)
    f.add_argument("--report", default=None)
    f.add_argument("--max-depth", type=int, default=6)
    f.add_argument("--min-samples-leaf", type=int, default=1)
    args = ap.parse_args(argv)
    if args.cmd == "run":
        run(args.first, args.count, args.out, args.reps, args.n_hi)
        return 0
    paths = [p for pat in args.records for p in sorted(glob.glob(pat))]
    recs = load(paths)
    rep, X, y = analyse(recs, args.max_depth, args.min_samples_leaf)
    print(json.dumps(rep, indent=1))
    if args.report:
        with open(args.report, "w") as fh:
            json.dump(rep, fh, indent=1)
    if args.model:
        from . import mo
        os.makedirs(os.path.dirname(os.path.abspath(args.model)), exist_ok=True)
        mo.write_model(args.model, [fitmod.fit_tree(X, y, args.max_depth, args.min_samples_leaf)])
    return 0


if __name__ == "__main__":
    sys.exit(main())
