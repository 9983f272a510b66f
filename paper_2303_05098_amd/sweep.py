"""Tuner sweep: the offline stage of the paper's pipeline (Section III-A) on synthetic
matrices.

    python -m paper_2303_05098_amd.sweep run --first 0 --count 64 --out sweep_000.jsonl     (GPU)
    python -m paper_2303_05098_amd.sweep features --first 0 --count 64 --out fe_000.jsonl     (GPU; feature time only)
    python -m paper_2303_05098_amd.sweep fit 'sweep_*.jsonl' --model paper_2303_05098_amd/models/mi355x_forest.bin

``run``: per matrix, features on the GPU (mo_features), then the run-first tuner (mo_tune, 1000 timed SpMVs per
feasible format as in Section VII-A); label = format with the smallest time.  ``fit``: the model-selection procedure
of Section VII-C (80 / 20 split, exhaustive grid search with 5-fold cross-validation for a decision tree and a
random forest, baseline against tuned, accuracy and balanced accuracy on the test set), geometric-mean speedup over
CSR of the true best and of the predicted format on the test set (SpMV only, and in the form of Eq. 2 with tuner
time included), tuner cost in CSR SpMVs (Section VII-D); the tuned forest, fitted on the training set, is written
as the model file mo_select loads.
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
NAMED_CONFIG_RECORDS = tuple(synth.SWEEP_BASE + 2 * i + 1 for i in range(4))   # configurations 1 .. 4 at full size


def run(first: int, count: int, out: str, reps: int, n_hi: float, ks=None) -> None:
    import torch

    from . import mo

    with open(out, "a") as fh:
        for k in (ks if ks is not None else range(first, first + count)):
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


def run_features(first: int, count: int, out: str, n_hi: float) -> None:
    """Feature-extraction time only (after a change to the feature kernels): lines {"k", "t_fe_ms", "features"} that
    `load` lays over the full records of the same matrices."""
    import torch

    from . import mo

    with open(out, "a") as fh:
        for k in range(first, first + count):
            fam, m, n, rp, ci, v = synth.sweep_matrix(k, 1e3, n_hi)
            a = mo.Csr(m, n, rp, ci, v)
            mo.mo_features(a)
            fe = []
            for _ in range(3):
                t0 = time.perf_counter()
                feats, ints = mo.mo_features(a)
                fe.append((time.perf_counter() - t0) * 1e3)
            fh.write(json.dumps(dict(k=k, t_fe_ms=min(fe), features=[float(f) for f in feats])) + "\n")
            fh.flush()
            if k % 64 == 0:
                print(f"[sweep features] k={k} {fam} m={m} t_fe={min(fe):.3f} ms", flush=True)
            del a
            torch.cuda.empty_cache()


def load(paths) -> list:
    """Records by matrix index; a later file wins.  Lines without timings (from `features`) only replace t_fe_ms, and
    must carry the same feature vector as the record they update."""
    recs, fe_only = {}, []
    for p in paths:
        for line in open(p):
            line = line.strip()
            if line:
                r = json.loads(line)
                if "ms_per_rep" in r:
                    recs[r["k"]] = r
                else:
                    fe_only.append(r)
    for r in fe_only:
        if r["k"] in recs:
            if recs[r["k"]]["features"] != r["features"]:
                raise ValueError(f"matrix {r['k']}: feature vector differs between the record and its update")
            recs[r["k"]]["t_fe_ms"] = r["t_fe_ms"]
    return [recs[k] for k in sorted(recs)]


def labels_with_tolerance(ms: np.ndarray, tol: float) -> np.ndarray:
    """Training label per matrix: the lowest format id among the formats whose time is within `tol` of the smallest
    (NaN = infeasible).  tol = 0 is the plain "format with the minimum runtime" of Section VII-A.  A small tolerance
    takes the timing jitter out of the labels where two formats run the very same kernel on the very same arrays (HDC
    whose diagonals are all true is DIA, HDC without a true diagonal is CSR, HYB whose ELL part holds every entry is
    ELL) or are launch-bound alike: the arg-min between such formats is noise, the lower id is as good a choice."""
    t = np.where(np.isnan(ms), np.inf, ms)
    tmin = t.min(axis=1, keepdims=True)
    ok = t <= tmin * (1.0 + tol)
    return np.argmax(ok, axis=1).astype(np.int64)


def geomean(v) -> float:
    v = np.asarray(v, dtype=np.float64)
    return float(np.exp(np.mean(np.log(v)))) if v.size else float("nan")


def _speedups(ms, t_fe, conv, y, pred, t_pred_ms, reps_eq2) -> dict:
    """Speedups over CSR and tuner cost for the rows given (Section VII-D / VII-E, Eq. 2)."""
    rows = np.arange(len(y))
    t_csr = ms[:, 1]
    t_best = ms[rows, y]
    # a predicted format that is infeasible for the matrix falls back to CSR, as a deployed tuner would
    t_sel = ms[rows, pred]
    t_sel = np.where(np.isnan(t_sel), t_csr, t_sel)
    t_min = np.nanmin(ms, axis=1)
    ratio = t_sel / t_min                        # how much slower the predicted format is than the fastest one
    rq = np.percentile(ratio, [50, 90, 99, 100])
    eq2 = (t_csr * reps_eq2) / (t_fe + t_pred_ms + t_sel * reps_eq2)
    cost = (t_fe + t_pred_ms) / t_csr
    q = np.percentile(cost, [0, 25, 50, 75, 100])
    # SpMVs after which tuning has paid for itself, conversion included (the paper leaves conversion out of Eq. 2):
    # smallest n with t_fe + t_pred + t_conv + n * t_sel < n * t_csr; only where the predicted format is faster
    t_conv = conv[rows, pred]
    gain = t_csr - t_sel
    pays = (gain > 0) & (pred != 1) & ~np.isnan(t_conv)
    breakeven = np.ceil((t_fe + t_pred_ms + t_conv)[pays] / gain[pays])
    bq = np.percentile(breakeven, [25, 50, 75]) if breakeven.size else [float("nan")] * 3
    return dict(
        n=int(len(y)),
        geomean_speedup_best_vs_csr=geomean(t_csr / t_best),
        geomean_speedup_predicted_vs_csr=geomean(t_csr / t_sel),
        geomean_speedup_eq2_predicted=geomean(eq2),
        predicted_over_fastest_time=dict(geomean=geomean(ratio), median=float(rq[0]), p90=float(rq[1]), p99=float(rq[2]),
                                         max=float(rq[3]), within_2_percent=float(np.mean(ratio <= 1.02)),
                                         within_5_percent=float(np.mean(ratio <= 1.05))),
        max_speedup_best_vs_csr=float(np.max(t_csr / t_best)),
        mean_speedup_best_vs_csr_where_not_csr=float(np.mean((t_csr / t_best)[y != 1])) if (y != 1).any() else None,
        tuner_cost_in_csr_spmv=dict(mean=float(cost.mean()), std=float(cost.std()), min=float(q[0]), q1=float(q[1]),
                                    q2=float(q[2]), q3=float(q[3]), max=float(q[4])),
        breakeven_spmvs_incl_conversion=dict(n_matrices=int(pays.sum()), q1=float(bq[0]), q2=float(bq[1]), q3=float(bq[2])))


def time_select(model, X, rounds: int = 20) -> float:
    """Host time of one mo_select with this model, in ms (T_PRED of Eq. 2), best of `rounds` passes over X."""
    from . import mo
    best = float("inf")
    for _ in range(rounds):
        t0 = time.perf_counter()
        mo.mo_predict(model, X)
        best = min(best, time.perf_counter() - t0)
    return best * 1e3 / max(1, len(X))


def analyse(recs, tree_grid=None, forest_grid=None, reps_eq2: int = 1000, score: str = "balanced_accuracy",
            tolerance: float = 0.0, label_tolerance: float = 0.02):
    """The procedure of Section VII-C on the records: stratified 80 / 20 split, grid search with 5-fold CV on the
    training set for a decision tree and a random forest, refit of the winners on the whole training set, accuracy
    and balanced accuracy of baseline and tuned models on the test set; then speedups over CSR and the tuner cost
    for the tuned forest on the test set (Sections VII-D, VII-E).  -> (report, tuned forest model, X, y, test mask)"""
    from . import mo
    X = np.array([r["features"] for r in recs], dtype=np.float64)
    ms = np.array([[np.nan if t is None else t for t in r["ms_per_rep"]] for r in recs], dtype=np.float64)
    conv = np.array([[np.nan if t is None else t for t in r["convert_ms"]] for r in recs], dtype=np.float64)
    t_fe = np.array([r["t_fe_ms"] for r in recs])
    y_strict = np.array([r["best"] for r in recs], dtype=np.int64)      # arg-min of the timings, as mo_tune returned it
    y = labels_with_tolerance(ms, label_tolerance)
    test = fitmod.train_test_split(y)
    Xtr, ytr, Xte, yte = X[~test], y[~test], X[test], y[test]

    def strip(e):
        return {k: v for k, v in e.items() if k != "pred"}

    out = dict(n=len(recs), n_train=int((~test).sum()), n_test=int(test.sum()),
               class_histogram={FORMATS[c]: int((y == c).sum()) for c in range(6)},
               class_histogram_strict_argmin={FORMATS[c]: int((y_strict == c).sum()) for c in range(6)},
               label_tolerance=label_tolerance, labels_changed_by_tolerance=int((y != y_strict).sum()),
               selection_score=score, selection_tolerance=tolerance)
    tuned = {}
    for kind, base, grid in (("tree", fitmod.BASELINE_TREE, tree_grid or fitmod.TREE_GRID),
                             ("forest", fitmod.BASELINE_FOREST, forest_grid or fitmod.FOREST_GRID)):
        gs = fitmod.grid_search(Xtr, ytr, grid, 5, score=score, tolerance=tolerance)
        cvb = fitmod.cross_validate(Xtr, ytr, 5, **base)
        eb = fitmod.evaluate(Xtr, ytr, Xte, yte, **base)
        et = fitmod.evaluate(Xtr, ytr, Xte, yte, **gs["best"])
        tuned[kind] = et
        out[kind] = dict(
            grid={k: list(v) for k, v in grid.items()}, grid_points=gs["n_points"],
            baseline=dict(cv_accuracy=cvb["accuracy"], cv_balanced_accuracy=cvb["balanced_accuracy"], test=strip(eb)),
            tuned=dict(cv_accuracy=gs["best_cv_accuracy"], cv_balanced_accuracy=gs["best_cv_balanced_accuracy"], test=strip(et)),
            top_cv_score=gs["top_cv_score"], best_by_score=gs["table"][:5])
    model = mo.mo_model_fit(Xtr, ytr, **out["forest"]["tuned"]["test"]["opts"])
    tree_model = mo.mo_model_fit(Xtr, ytr, **out["tree"]["tuned"]["test"]["opts"])
    t_pred = time_select(model, X)
    out["t_pred_ms"] = dict(tuned_forest=t_pred, tuned_tree=time_select(tree_model, X))
    out["predicted_histogram_test"] = {FORMATS[c]: int((tuned["forest"]["pred"] == c).sum()) for c in range(6)}
    out["test_set_tuned_forest"] = _speedups(ms[test], t_fe[test], conv[test], yte, tuned["forest"]["pred"], t_pred, reps_eq2)
    out["test_set_tuned_tree"] = _speedups(ms[test], t_fe[test], conv[test], yte, tuned["tree"]["pred"],
                                           out["t_pred_ms"]["tuned_tree"], reps_eq2)
    out["all_records_oracle_choice"] = _speedups(ms, t_fe, conv, y, y, t_pred, reps_eq2)
    out["test_set_tuned_forest"]["accuracy_vs_strict_argmin"] = fitmod.accuracy(y_strict[test], tuned["forest"]["pred"])
    # the four benchmark configurations at their own size, when the records hold them: what the committed model says
    # (they may lie in the training set: this is a statement about the model file, not a generalisation score)
    pred_all = mo.mo_predict(model, X)
    named = []
    for i, r in enumerate(recs):
        if str(r.get("family", "")).startswith("config") and r["k"] in NAMED_CONFIG_RECORDS:
            t = ms[i]
            tp = t[pred_all[i]] if not np.isnan(t[pred_all[i]]) else t[1]
            named.append(dict(k=r["k"], family=r["family"], m=r["m"], nnz=r["nnz"], in_test_set=bool(test[i]),
                              fastest=FORMATS[int(np.nanargmin(t))], predicted=FORMATS[int(pred_all[i])],
                              predicted_over_fastest_time=float(tp / np.nanmin(t)),
                              us_per_format={FORMATS[c]: (None if np.isnan(t[c]) else round(float(t[c]) * 1e3, 2)) for c in range(6)}))
    out["benchmark_configurations"] = named
    tree_model.free()
    return out, model, X, y, test


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    r = sub.add_parser("run")
    r.add_argument("--first", type=int, default=0)
    r.add_argument("--count", type=int, default=256)
    r.add_argument("--out", required=True)
    r.add_argument("--reps", type=int, default=1000)
    r.add_argument("--n-hi", type=float, default=4e6)
    r.add_argument("--ks", default=None, help="comma-separated matrix indices to run instead of --first / --count (re-runs of single records)")
    q = sub.add_parser("features")
    q.add_argument("--first", type=int, default=0)
    q.add_argument("--count", type=int, default=256)
    q.add_argument("--out", required=True)
    q.add_argument("--n-hi", type=float, default=4e6)
    f = sub.add_parser("fit")
    f.add_argument("records", nargs="+")
    f.add_argument("--model", default=None)
    f.add_argument("--report", default=None)
    f.add_argument("--score", default="balanced_accuracy", choices=["accuracy", "balanced_accuracy"])
    f.add_argument("--tolerance", type=float, default=0.0,
                   help="pick the cheapest model whose CV score is within this much of the best one")
    f.add_argument("--label-tolerance", type=float, default=0.02,
                   help="training label = lowest format id among the formats within this fraction of the fastest time (0 = plain arg-min)")
    f.add_argument("--grid", default=None, help="JSON file {\"tree\": {...}, \"forest\": {...}} replacing the built-in grids")
    args = ap.parse_args(argv)
    if args.cmd == "run":
        run(args.first, args.count, args.out, args.reps, args.n_hi, [int(t) for t in args.ks.split(",")] if args.ks else None)
        return 0
    if args.cmd == "features":
        run_features(args.first, args.count, args.out, args.n_hi)
        return 0
    paths = [p for pat in args.records for p in sorted(glob.glob(pat))]
    recs = load(paths)
    grids = json.load(open(args.grid)) if args.grid else {}
    rep, model, X, y, test = analyse(recs, grids.get("tree"), grids.get("forest"), score=args.score, tolerance=args.tolerance,
                                      label_tolerance=args.label_tolerance)
    print(json.dumps(rep, indent=1))
    if args.report:
        with open(args.report, "w") as fh:
            json.dump(rep, fh, indent=1)
    if args.model:
        from . import mo
        os.makedirs(os.path.dirname(os.path.abspath(args.model)), exist_ok=True)
        mo.mo_model_save(model, args.model)
    return 0


if __name__ == "__main__":
    sys.exit(main())
