"""Host-side training of the format classifier (Section V and VII-C of the paper: a decision tree over the ten
features, evaluated with 5-fold cross-validation; accuracy and balanced accuracy as in Section VII-C).

Plain numpy CART, written for a few hundred samples:
  * criterion gini, threshold = midpoint between consecutive distinct values of a feature,
  * best split = lowest weighted impurity; ties -> lowest feature index, then lowest threshold,
  * a node becomes a leaf when it is pure, at max_depth, smaller than 2 * min_samples_leaf, or has no valid split,
  * leaf class = majority of the training samples at the leaf, ties -> lowest class id.
The tree comes out in the array layout of the binary model file (children after their parent), ready for
``mo.write_model``.  Nothing here runs on the GPU.
"""
from __future__ import annotations

import numpy as np

from . import synth

N_CLASSES = 6


def _gini_from_counts(counts: np.ndarray) -> np.ndarray:
    tot = counts.sum(axis=-1)
    with np.errstate(divide="ignore", invalid="ignore"):
        g = 1.0 - ((counts / tot[..., None]) ** 2).sum(axis=-1)
    return np.where(tot > 0, g, 0.0)


def _best_split(X: np.ndarray, y: np.ndarray, min_leaf: int):
    n, nf = X.shape
    best = None   # (impurity, feature, threshold)
    onehot = np.eye(N_CLASSES)[y]
    for f in range(nf):
        order = np.argsort(X[:, f], kind="stable")
        xs = X[order, f]
        left = np.cumsum(onehot[order], axis=0)            # counts with the first i+1 samples on the left
        total = left[-1]
        cut = np.nonzero(xs[1:] > xs[:-1])[0]              # split between i and i+1
        if min_leaf > 1:
            cut = cut[(cut + 1 >= min_leaf) & (n - cut - 1 >= min_leaf)]
        if cut.size == 0:
            continue
        lc = left[cut]
        rc = total[None, :] - lc
        nl = (cut + 1).astype(np.float64)
        nr = n - nl
        imp = (nl * _gini_from_counts(lc) + nr * _gini_from_counts(rc)) / n
        i = int(np.argmin(imp))                            # first minimum = lowest threshold on ties
        cand = (float(imp[i]), f, 0.5 * (float(xs[cut[i]]) + float(xs[cut[i] + 1])))
        if best is None or cand[0] < best[0] - 1e-15:
            best = cand
    return best


def fit_tree(X, y, max_depth: int = 6, min_samples_leaf: int = 1) -> dict:
    """-> dict(feature, threshold, left, right, klass) in model-file layout."""
    X = np.asarray(X, dtype=np.float64)
    y = np.asarray(y, dtype=np.int64)
    feature, threshold, left, right, klass = [], [], [], [], []

    def grow(idx: np.ndarray, depth: int) -> int:
        me = len(feature)
        counts = np.bincount(y[idx], minlength=N_CLASSES)
        feature.append(-1); threshold.append(0.0); left.append(-1); right.append(-1); klass.append(int(np.argmax(counts)))
        if depth >= max_depth or np.count_nonzero(counts) <= 1 or idx.size < 2 * min_samples_leaf:
            return me
        split = _best_split(X[idx], y[idx], min_samples_leaf)
        if split is None:
            return me
        _, f, t = split
        go_left = X[idx, f] <= t
        feature[me], threshold[me], klass[me] = f, t, -1
        left[me] = grow(idx[go_left], depth + 1)
        right[me] = grow(idx[~go_left], depth + 1)
        return me

    grow(np.arange(X.shape[0]), 0)
    return dict(feature=feature, threshold=threshold, left=left, right=right, klass=klass)


def predict_tree(tree: dict, X) -> np.ndarray:
    """Host prediction for training-time bookkeeping (the deployed path is mo_select in the library)."""
    X = np.asarray(X, dtype=np.float64)
    out = np.zeros(X.shape[0], dtype=np.int64)
    for i, x in enumerate(X):
        node = 0
        while tree["feature"][node] >= 0:
            node = tree["left"][node] if x[tree["feature"][node]] <= tree["threshold"][node] else tree["right"][node]
        out[i] = tree["klass"][node]
    return out


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


def accuracy(y_true, y_pred) -> float:
    y_true, y_pred = np.asarray(y_true), np.asarray(y_pred)
    return float(np.mean(y_true == y_pred)) if y_true.size else float("nan")


def balanced_accuracy(y_true, y_pred) -> float:
    """Mean over the classes present in y_true of the per-class recall (Section VII-C)."""
    y_true, y_pred = np.asarray(y_true), np.asarray(y_pred)
    rec = [float(np.mean(y_pred[y_true == c] == c)) for c in np.unique(y_true)]
    return float(np.mean(rec)) if rec else float("nan")


def cross_validate(X, y, k: int = 5, max_depth: int = 6, min_samples_leaf: int = 1, seed: int = synth.BASE_SEED) -> dict:
    X = np.asarray(X, dtype=np.float64)
    y = np.asarray(y, dtype=np.int64)
    fold = stratified_folds(y, k, seed)
    pred = np.zeros_like(y)
    per_fold = []
    for j in range(k):
        tr, te = fold != j, fold == j
        if not te.any() or not tr.any():
            continue
        tree = fit_tree(X[tr], y[tr], max_depth, min_samples_leaf)
        pred[te] = predict_tree(tree, X[te])
        per_fold.append(dict(fold=j, n=int(te.sum()), accuracy=accuracy(y[te], pred[te]),
                             balanced_accuracy=balanced_accuracy(y[te], pred[te])))
    return dict(pred=pred, fold=fold, per_fold=per_fold, accuracy=accuracy(y, pred), balanced_accuracy=balanced_accuracy(y, pred))
