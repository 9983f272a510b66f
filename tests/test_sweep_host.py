"""Sweep bookkeeping on the CPU: the committed MI355X records load, the analysis identities hold, the committed
model file is what a refit of those records gives."""
import json
import math
import os

import numpy as np

from paper_2303_05098_amd import fit, mo, sweep

MODELS = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2303_05098_amd", "models")


def test_committed_records_and_identities():
    recs = sweep.load([os.path.join(MODELS, "mi355x_sweep.jsonl")])
    assert len(recs) == 256 and [r["k"] for r in recs] == list(range(256))
    for r in recs:
        ms = [math.nan if t is None else t for t in r["ms_per_rep"]]
        assert r["best"] == mo.mo_pick(ms)                      # label = argmin of the timings (Section VII-A)
        assert not math.isnan(ms[0]) and not math.isnan(ms[1]) and not math.isnan(ms[4]) and not math.isnan(ms[5])
        assert len(r["features"]) == 10 and r["features"][2] == r["nnz"]
    rep, X, y = sweep.analyse(recs, 6, 1)
    assert sum(rep["class_histogram"].values()) == 256
    assert rep["geomean_speedup_best_vs_csr"] >= 1.0            # the best format is never slower than CSR
    assert rep["geomean_speedup_predicted_vs_csr"] <= rep["geomean_speedup_best_vs_csr"] + 1e-12
    assert 0.0 <= rep["cv_balanced_accuracy"] <= 1.0 and 0.0 <= rep["cv_accuracy"] <= 1.0
    saved = json.load(open(os.path.join(MODELS, "mi355x_sweep_report.json")))
    assert abs(saved["cv_accuracy"] - rep["cv_accuracy"]) < 1e-12


def test_committed_model_matches_refit(tmp_path):
    recs = sweep.load([os.path.join(MODELS, "mi355x_sweep.jsonl")])
    X = np.array([r["features"] for r in recs])
    y = np.array([r["best"] for r in recs])
    tree = fit.fit_tree(X, y, 6, 1)
    p = str(tmp_path / "m.bin")
    mo.write_model(p, [tree])
    assert open(p, "rb").read() == open(os.path.join(MODELS, "mi355x_tree.bin"), "rb").read()
    mdl = mo.mo_model_load(os.path.join(MODELS, "mi355x_tree.bin"))
    pred = fit.predict_tree(tree, X)
    assert [mo.mo_select(mdl, x) for x in X] == list(pred)
