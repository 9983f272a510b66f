"""Model selection around the library's host trainer (Section VII-C): stratified train / test split and folds,
accuracy and balanced accuracy, 5-fold cross-validation and the exhaustive grid search over the hyper-parameters of
Table III.  Trees and forests are fitted by ``mo.mo_model_fit`` and evaluated by ``mo.mo_predict`` (native host code
in the library); this module only deals rows to folds, loops over the grid and counts hits.
"""
from __future__ import annotations

import itertools
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from . import mo, synth

N_CLASSES = 6

# Baseline column of Table III (scikit-learn's defaults at the time: 100 estimators, bootstrap, unlimited depth).
BASELINE_FOREST = dict(n_estimators=100, bootstrap=1, max_depth=-1, min_samples_leaf=1, min_samples_split=2,
                       max_features=10, criterion="gini")
BASELINE_TREE = dict(n_estimators=1, bootstrap=0, max_depth=-1, min_samples_leaf=1, min_samples_split=2,
                     max_features=10, criterion="gini")

# Search space: the ranges the tuned column of Table III spans (20-90 estimators, depth 10-21, leaf 1-3, split
# 2 / 5 / 10, 4-10 features, both criteria, with and without bootstrap), thinned to a grid that one host searches
# in about a minute on a few hundred records.
FOREST_GRID = dict(n_estimators=[20, 50, 100], bootstrap=[0, 1], max_depth=[5, 10, 15, -1],
                   min_samples_leaf=[1, 2, 3], min_samples_split=[2, 10], max_features=[4, 7, 10],
                   criterion=["gini", "entropy"])
TREE_GRID = dict(n_estimators=[1], bootstrap=[0], max_depth=[2, 3, 4, 5, 6, 8, 10, 12, 16, 20, -1],
                 min_samples_leaf=[1, 2, 3, 5, 8], min_samples_split=[2, 5, 10, 20], max_features=[10],
                 criterion=["gini", "entropy"])


def stratified_folds(y, k: int = 5, seed: int = synth.BASE_SEED) -> np.ndarray:
    """fold id per sample: inside every class the samples are shuffled by a seeded hash and dealt round-robin."""
    y = np.asarray(y, dtype=np.int64)
    fold = np.zeros(y.shape[0], dtype=np.int64)
    start = 0
    for c in range(N_CLASSES):
        idx = np.nonzero(y == c)[0]
        order = idx[np.argsort(synth.uniform01(seed, 900 + c, idx), kind="stable")]
        fold[order] = (start + np.arange(order.size)) % k
        start += order.size
    return fold


def train_test_split(y, test_every: int = 5, seed: int = synth.BASE_SEED + 1) -> np.ndarray:
    """Boolean mask of the test set: a stratified 1 / test_every share (80 % / 20 % as in Section VII "Setup")."""
    return stratified_folds(y, test_every, seed) == 0


def accuracy(y_true, y_pred) -> float:
    y_true, y_pred = np.asarray(y_true), np.asarray(y_pred)
    return float(np.mean(y_true == y_pred)) if y_true.size else float("nan")


def balanced_accuracy(y_true, y_pred) -> float:
    """Mean over the classes present in y_true of the per-class recall (Section VII-C)."""
    y_true, y_pred = np.asarray(y_true), np.asarray(y_pred)
    rec = [float(np.mean(y_pred[y_true == c] == c)) for c in np.unique(y_true)]
    return float(np.mean(rec)) if rec else float("nan")


def fit(X, y, seed: int = 0, **opts) -> "mo.Model":
    return mo.mo_model_fit(X, y, seed=seed, **opts)


def cross_validate(X, y, k: int = 5, seed: int = synth.BASE_SEED, fold=None, **opts) -> dict:
    """k-fold CV of one hyper-parameter setting: every sample is predicted by the model that did not see it."""
    X = np.asarray(X, dtype=np.float64)
    y = np.asarray(y, dtype=np.int64)
    fold = stratified_folds(y, k, seed) if fold is None else fold
    pred = np.zeros_like(y)
    per_fold = []
    for j in range(k):
        tr, te = fold != j, fold == j
        if not te.any() or not tr.any():
            continue
        model = mo.mo_model_fit(X[tr], y[tr], seed=seed + j, **opts)
        pred[te] = mo.mo_predict(model, X[te])
        model.free()
        per_fold.append(dict(fold=j, n=int(te.sum()), accuracy=accuracy(y[te], pred[te]),
                             balanced_accuracy=balanced_accuracy(y[te], pred[te])))
    return dict(pred=pred, fold=fold, per_fold=per_fold, accuracy=accuracy(y, pred), balanced_accuracy=balanced_accuracy(y, pred))


def grid_points(grid: dict) -> list:
    keys = list(grid)
    return [dict(zip(keys, vals)) for vals in itertools.product(*(grid[k] for k in keys))]


def model_cost(o: dict) -> tuple:
    """Prediction cost proxy used to break score ties: fewer trees, then shallower (unlimited counts as deepest)."""
    return (o["n_estimators"], 1 << 30 if o["max_depth"] < 0 else o["max_depth"])


def grid_search(X, y, grid: dict, k: int = 5, seed: int = synth.BASE_SEED, score: str = "balanced_accuracy",
                workers: int | None = None, tolerance: float = 0.0) -> dict:
    """Exhaustive search (Section VII-C): the whole k-fold CV for every grid point, on the same folds.  The winner is
    the cheapest model (fewest trees, then shallowest, then the earlier grid point) among the points whose
    mean-over-samples `score` is within `tolerance` of the highest one; tolerance 0 is the plain arg-max with ties to
    the cheaper model."""
    X = np.asarray(X, dtype=np.float64)
    y = np.asarray(y, dtype=np.int64)
    fold = stratified_folds(y, k, seed)
    points = grid_points(grid)

    def one(o):
        cv = cross_validate(X, y, k, seed, fold, **o)
        return cv["accuracy"], cv["balanced_accuracy"]

    # the trainer is native code called through ctypes, which releases the interpreter lock: threads scale
    with ThreadPoolExecutor(max_workers=workers or min(16, os.cpu_count() or 1)) as ex:
        scores = list(ex.map(one, points))
    col = 1 if score == "balanced_accuracy" else 0
    order = sorted(range(len(points)), key=lambda i: (-scores[i][col], model_cost(points[i]), i))
    top = scores[order[0]][col]
    best = min((i for i in order if scores[i][col] >= top - tolerance), key=lambda i: (model_cost(points[i]), -scores[i][col], i))
    return dict(best=points[best], best_cv_accuracy=scores[best][0], best_cv_balanced_accuracy=scores[best][1],
                top_cv_score=top, tolerance=tolerance, n_points=len(points), score=score,
                table=[dict(opts=points[i], cv_accuracy=scores[i][0], cv_balanced_accuracy=scores[i][1]) for i in order])


def evaluate(X_train, y_train, X_test, y_test, seed: int = 0, **opts) -> dict:
    """Fit on the full training set, score on the held-out test set (the two score columns of Table III)."""
    model = mo.mo_model_fit(X_train, y_train, seed=seed, **opts)
    pred = mo.mo_predict(model, X_test)
    nt, nn = model.info()
    model.free()
    return dict(opts=opts, accuracy=accuracy(y_test, pred), balanced_accuracy=balanced_accuracy(y_test, pred),
                n_trees=nt, n_nodes=nn, pred=pred)
