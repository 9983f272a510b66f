"""Sweep bookkeeping on the CPU: the committed MI355X records load, the analysis identities hold, and the committed
report and model file are what the committed records give (refits of the reported settings, not a new search)."""
import json
import math
import os

import numpy as np

from paper_2303_05098_amd import fit, mo, sweep

MODELS = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2303_05098_amd", "models")


def records():
    return sweep.load([os.path.join(MODELS, "mi355x_sweep.jsonl")])


def report():
    return json.load(open(os.path.join(MODELS, "mi355x_sweep_report.json")))


def arrays(recs):
    """Features and training labels as `sweep fit` forms them: label = lowest id within the reported tolerance of the
    fastest format."""
    X = np.array([r["features"] for r in recs], dtype=np.float64)
    ms = np.array([[np.nan if t is None else t for t in r["ms_per_rep"]] for r in recs], dtype=np.float64)
    y = sweep.labels_with_tolerance(ms, report()["label_tolerance"])
    return X, y


def test_committed_records():
    recs = records()
    assert len(recs) == 2560 and [r["k"] for r in recs] == list(range(2560))
    assert sum(r["family"] == "banded_clustered" for r in recs) == 256
    assert [r["family"] for r in recs if r["k"] in sweep.NAMED_CONFIG_RECORDS] == ["config%d_scaled" % c for c in (1, 2, 3, 4)]
    for r in recs:
        ms = [math.nan if t is None else t for t in r["ms_per_rep"]]
        assert r["best"] == mo.mo_pick(ms)                      # label = argmin of the timings (Section VII-A)
        assert not math.isnan(ms[0]) and not math.isnan(ms[1]) and not math.isnan(ms[4]) and not math.isnan(ms[5])
        assert len(r["features"]) == 10 and r["features"][2] == r["nnz"] and r["reps"] == 1000


def test_committed_report_is_what_the_records_give():
    recs = records()
    X, y = arrays(recs)
    rep = json.load(open(os.path.join(MODELS, "mi355x_sweep_report.json")))
    test = fit.train_test_split(y)
    assert (rep["n"], rep["n_train"], rep["n_test"]) == (2560, int((~test).sum()), int(test.sum()))
    assert abs(rep["n_test"] / rep["n"] - 0.2) < 0.005
    assert sum(rep["class_histogram"].values()) == 2560
    assert rep["class_histogram"] == {sweep.FORMATS[c]: int((y == c).sum()) for c in range(6)}
    strict = np.array([r["best"] for r in recs])
    assert rep["labels_changed_by_tolerance"] == int((y != strict).sum())
    for kind, base in (("tree", fit.BASELINE_TREE), ("forest", fit.BASELINE_FOREST)):
        assert rep[kind]["baseline"]["test"]["opts"] == base
        for which in ("baseline", "tuned"):
            want = rep[kind][which]["test"]
            got = fit.evaluate(X[~test], y[~test], X[test], y[test], **want["opts"])
            assert (got["accuracy"], got["balanced_accuracy"], got["n_trees"], got["n_nodes"]) == \
                (want["accuracy"], want["balanced_accuracy"], want["n_trees"], want["n_nodes"])
        # the tuned setting is a point of the reported grid and won the search by the reported score
        tuned = rep[kind]["tuned"]
        assert all(tuned["test"]["opts"][k] in rep[kind]["grid"][k] for k in rep[kind]["grid"])
        # ... and won the search: within the tolerance of the best score, and none of the higher-scoring points is cheaper
        top, tol = rep[kind]["top_cv_score"], rep["selection_tolerance"]
        assert rep[kind]["best_by_score"][0]["cv_balanced_accuracy"] == top
        assert top - tol <= tuned["cv_balanced_accuracy"] <= top
        for r in rep[kind]["best_by_score"]:
            if r["cv_balanced_accuracy"] >= top - tol:
                assert fit.model_cost(tuned["test"]["opts"]) <= fit.model_cost(r["opts"])
        cv = fit.cross_validate(X[~test], y[~test], 5, **tuned["test"]["opts"])
        assert (cv["accuracy"], cv["balanced_accuracy"]) == (tuned["cv_accuracy"], tuned["cv_balanced_accuracy"])
    # speedups on the test set: the best format is never slower than CSR, a prediction never beats the best
    for key in ("test_set_tuned_forest", "test_set_tuned_tree", "all_records_oracle_choice"):
        s = rep[key]
        assert s["geomean_speedup_best_vs_csr"] >= 1.0
        assert s["geomean_speedup_predicted_vs_csr"] <= s["geomean_speedup_best_vs_csr"] + 1e-12
        assert s["geomean_speedup_eq2_predicted"] <= s["geomean_speedup_predicted_vs_csr"]      # tuner time only adds
    o = rep["all_records_oracle_choice"]
    assert o["geomean_speedup_predicted_vs_csr"] == o["geomean_speedup_best_vs_csr"]


def test_speedup_bookkeeping_on_a_hand_case():
    ms = np.array([[4.0, 2.0, 1.0, np.nan, 3.0, 2.0], [1.0, 2.0, np.nan, np.nan, 4.0, 8.0]])
    conv = np.full((2, 6), 10.0)
    s = sweep._speedups(ms, np.array([1.0, 1.0]), conv, np.array([2, 0]), np.array([2, 3]), 0.5, 1000)
    # row 0 predicted DIA (2x faster than CSR); row 1 predicted ELL, infeasible -> falls back to CSR (1x)
    assert abs(s["geomean_speedup_predicted_vs_csr"] - math.sqrt(2.0 * 1.0)) < 1e-12
    assert abs(s["geomean_speedup_best_vs_csr"] - 2.0) < 1e-12
    assert abs(s["geomean_speedup_eq2_predicted"] - math.sqrt((2000 / 1001.5) * (2000 / 2001.5))) < 1e-12
    assert abs(s["tuner_cost_in_csr_spmv"]["mean"] - 0.75) < 1e-12                 # (1 + 0.5) / 2 for both rows
    # break-even only where the prediction is faster than CSR: (1 + 0.5 + 10) / (2 - 1) -> 12 SpMVs
    assert s["breakeven_spmvs_incl_conversion"] == dict(n_matrices=1, q1=12.0, q2=12.0, q3=12.0)


def test_committed_model_is_the_tuned_forest_fitted_on_the_training_set(tmp_path):
    recs = records()
    X, y = arrays(recs)
    rep = json.load(open(os.path.join(MODELS, "mi355x_sweep_report.json")))
    test = fit.train_test_split(y)
    model = mo.mo_model_fit(X[~test], y[~test], **rep["forest"]["tuned"]["test"]["opts"])
    p = str(tmp_path / "m.bin")
    mo.mo_model_save(model, p)
    committed = os.path.join(MODELS, "mi355x_forest.bin")
    assert open(p, "rb").read() == open(committed, "rb").read()
    loaded = mo.mo_model_load(committed)
    assert np.array_equal(mo.mo_predict(loaded, X), mo.mo_predict(model, X))
    assert fit.accuracy(y[test], mo.mo_predict(loaded, X[test])) == rep["forest"]["tuned"]["test"]["accuracy"]


def test_feature_time_updates_lay_over_records(tmp_path):
    """Lines written by `sweep features` replace t_fe_ms of the record with the same k, whatever the file order, and a
    line whose feature vector differs from the record's is refused."""
    full = dict(k=3, family="x", m=2, n=2, nnz=2, features=[2.0] * 10, t_fe_ms=1.0, ms_per_rep=[1.0] * 6, convert_ms=[0.1] * 6,
                best=1, reps=1000)
    other = dict(full, k=4, t_fe_ms=2.0)
    a, b = tmp_path / "a.jsonl", tmp_path / "b.jsonl"
    a.write_text(json.dumps(dict(k=3, t_fe_ms=0.25, features=[2.0] * 10)) + "\n" + json.dumps(dict(k=9, t_fe_ms=0.5, features=[1.0] * 10)) + "\n")
    b.write_text(json.dumps(full) + "\n" + json.dumps(other) + "\n")
    for order in ([a, b], [b, a]):
        recs = sweep.load([str(p) for p in order])
        assert [r["k"] for r in recs] == [3, 4] and [r["t_fe_ms"] for r in recs] == [0.25, 2.0]
        assert recs[0]["ms_per_rep"] == [1.0] * 6
    a.write_text(json.dumps(dict(k=3, t_fe_ms=0.25, features=[3.0] * 10)) + "\n")
    import pytest
    with pytest.raises(ValueError):
        sweep.load([str(a), str(b)])


def test_labels_with_tolerance():
    """The training label is the lowest id among the formats within the tolerance of the fastest; infeasible formats
    never win; tolerance 0 is mo_pick."""
    ms = np.array([[4.0, 2.0, 1.0, np.nan, 3.0, 1.01],       # DIA and HDC within 2 %: DIA (lower id)
                   [1.0, 2.0, np.nan, np.nan, 0.99, 8.0],     # HYB fastest, COO within 2 %: COO
                   [np.nan, 5.0, np.nan, np.nan, np.nan, 5.0],  # exact tie CSR / HDC: CSR
                   [3.0, 2.0, 1.0, 1.5, 1.021, 1.03]])        # nothing within 2 % of DIA but DIA
    assert sweep.labels_with_tolerance(ms, 0.02).tolist() == [2, 0, 1, 2]
    strict = sweep.labels_with_tolerance(ms, 0.0)
    assert strict.tolist() == [mo.mo_pick(row) for row in ms] == [2, 4, 1, 2]
    # never slower than (1 + tol) times the fastest
    t = np.where(np.isnan(ms), np.inf, ms)
    lab = sweep.labels_with_tolerance(ms, 0.02)
    assert np.all(t[np.arange(4), lab] <= 1.02 * t.min(axis=1))


def test_extra_sweep_matrices():
    """Indices 2048 .. 2559: clustered bands on even indices, the benchmark configurations on odd ones (the first four at
    their own size); every other index keeps the five rotating families."""
    from paper_2303_05098_amd import synth
    fam, m, n, rp, ci, v = synth.sweep_matrix(2052, 1e3, 2e4)
    assert fam == "banded_clustered" and m == n
    d = np.unique(ci.astype(np.int64) - np.repeat(np.arange(m), np.diff(rp)))
    cnt = np.bincount(ci.astype(np.int64) - np.repeat(np.arange(m), np.diff(rp)) + m - 1, minlength=2 * m - 1)
    full = np.nonzero(cnt * 2 >= m)[0] - (m - 1)                 # the band: diagonals populated over more than half their length
    assert 0 in full and np.array_equal(full, -full[::-1])       # symmetric clusters around the main diagonal
    assert d.size >= full.size
    assert synth.sweep_matrix(2049)[0] == "config1_scaled" and synth.sweep_matrix(2049)[1] == 4096
    fam, m = synth.sweep_matrix(2065, 1e3, 2e4)[:2]
    assert fam == "config1_scaled" and m != 4096
    assert synth.sweep_matrix(2560, 1e3, 2e4)[0] == synth.FAMILIES[2560 % 5]
    assert synth.sweep_matrix(5003, 1e3, 2e4)[0] == synth.FAMILIES[5003 % 5]
    a, b = synth.sweep_matrix(2052, 1e3, 2e4), synth.sweep_matrix(2052, 1e3, 2e4)
    assert all(np.array_equal(x, y) for x, y in zip(a[3:], b[3:]))
