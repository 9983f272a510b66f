"""Model selection on the host: folds, split, metrics (pinned against scikit-learn's metric and hand values), and
the grid search's bookkeeping (same folds for every point, winner = best score, ties to the cheaper model)."""
import numpy as np
import pytest

from oracle import cart
from paper_2303_05098_amd import fit, mo, synth
from tests.test_oracle_cart import data


def test_stratified_folds_split_and_metrics():
    y = np.array([1] * 50 + [2] * 10 + [5] * 5)
    fold = fit.stratified_folds(y, 5)
    for c, n in ((1, 50), (2, 10), (5, 5)):
        cnt = np.bincount(fold[y == c], minlength=5)
        assert cnt.sum() == n and cnt.max() - cnt.min() <= 1
    assert np.bincount(fold, minlength=5).max() - np.bincount(fold, minlength=5).min() <= 1
    test = fit.train_test_split(y)
    assert test.sum() == 13 and [int(test[y == c].sum()) for c in (1, 2, 5)] == [10, 2, 1]      # 20 % of every class
    assert not np.array_equal(test, fold == 0)                                                   # split and folds use different draws
    assert fit.accuracy([1, 1, 2, 5], [1, 2, 2, 5]) == 0.75
    # recalls: class 1 -> 1/2, class 2 -> 1, class 5 -> 1
    assert abs(fit.balanced_accuracy([1, 1, 2, 5], [1, 2, 2, 5]) - (0.5 + 1 + 1) / 3) < 1e-15
    from sklearn.metrics import balanced_accuracy_score
    yt = (synth.uniform01(1, 0, np.arange(200)) * 4).astype(int)
    yp = (synth.uniform01(2, 0, np.arange(200)) * 4).astype(int)
    assert abs(fit.balanced_accuracy(yt, yp) - balanced_accuracy_score(yt, yp)) < 1e-12


def test_cross_validation_predicts_every_sample_with_a_model_that_did_not_see_it():
    X, y = data(6, 150, noise=0.1)
    opts = dict(n_estimators=3, bootstrap=1, max_depth=5, min_samples_leaf=1, min_samples_split=2, max_features=4, criterion="gini")
    cv = fit.cross_validate(X, y, 5, seed=77, **opts)
    assert len(cv["per_fold"]) == 5 and sum(f["n"] for f in cv["per_fold"]) == 150
    # the same thing by hand, with the oracle trainer
    fold = fit.stratified_folds(y, 5, 77)
    want = np.zeros_like(y)
    for j in range(5):
        o = cart.Opts(seed=77 + j, **{**opts, "bootstrap": True})
        trees = cart.fit_forest(X[fold != j], y[fold != j], o)
        want[fold == j] = cart.predict(trees, X[fold == j])
    assert np.array_equal(cv["pred"], want)
    assert cv["accuracy"] == np.mean(want == y)


def test_grid_search_bookkeeping():
    X, y = data(8, 160, noise=0.2)
    grid = dict(n_estimators=[1, 5], bootstrap=[0, 1], max_depth=[1, 4, -1], min_samples_leaf=[1, 4], min_samples_split=[2],
                max_features=[3, 10], criterion=["gini", "entropy"])
    gs = fit.grid_search(X, y, grid, 5, seed=5, workers=4)
    assert gs["n_points"] == 2 * 2 * 3 * 2 * 2 * 2 == len(gs["table"])
    scores = [r["cv_balanced_accuracy"] for r in gs["table"]]
    assert scores == sorted(scores, reverse=True) and gs["best"] == gs["table"][0]["opts"]
    # every row is what cross_validate gives for that point on the same folds, whatever thread ran it
    for r in gs["table"][::7]:
        cv = fit.cross_validate(X, y, 5, seed=5, **r["opts"])
        assert (cv["accuracy"], cv["balanced_accuracy"]) == (r["cv_accuracy"], r["cv_balanced_accuracy"])
    # ties go to the cheaper model: with a constant label every point scores 1.0 and the smallest forest wins
    gc = fit.grid_search(X, np.full(160, 3), grid, 5, workers=2)
    assert gc["best_cv_accuracy"] == 1.0 and gc["best"]["n_estimators"] == 1 and gc["best"]["max_depth"] == 1
    # a tolerance trades score for a cheaper model: the winner is the cheapest point within it
    gt = fit.grid_search(X, y, grid, 5, seed=5, workers=4, tolerance=0.05)
    top = gt["table"][0]["cv_balanced_accuracy"]
    assert gt["top_cv_score"] == top and top - 0.05 <= gt["best_cv_balanced_accuracy"] <= top
    within = [r["opts"] for r in gt["table"] if r["cv_balanced_accuracy"] >= top - 0.05]
    assert fit.model_cost(gt["best"]) == min(fit.model_cost(o) for o in within)
    assert fit.model_cost(gt["best"]) <= fit.model_cost(gs["best"])
    # selection by plain accuracy
    ga = fit.grid_search(X, y, grid, 5, seed=5, score="accuracy", workers=4)
    acc = [r["cv_accuracy"] for r in ga["table"]]
    assert acc == sorted(acc, reverse=True)


def test_evaluate_and_tuning_helps_on_noisy_labels():
    X, y = data(9, 400, noise=0.25)
    test = fit.train_test_split(y)
    base = fit.evaluate(X[~test], y[~test], X[test], y[test], **fit.BASELINE_TREE)
    shallow = fit.evaluate(X[~test], y[~test], X[test], y[test], **{**fit.BASELINE_TREE, "max_depth": 5, "min_samples_leaf": 5})
    assert base["n_trees"] == 1 and shallow["n_nodes"] < base["n_nodes"]
    assert shallow["accuracy"] >= base["accuracy"]                 # an unlimited tree fits the label noise
    assert len(base["pred"]) == test.sum()
