"""CPU oracle of the offline training stage: CART decision trees and random forests over the ten features
(Section V "decision tree ... ensemble of decision trees", Section VII-C hyper-parameters of Table III: number of
estimators, bootstrap, max depth, min samples per leaf, min samples before a split, max features per split,
criterion gini / entropy).

TEST INFRASTRUCTURE ONLY: slow, plain Python loops over small data, exact integers where the arithmetic allows.
Imported by tests (and by nothing in the product); shares no code with the C++ trainer in the library.

The algorithm, step by step (the paper names scikit-learn's classifiers and gives no listing, so the steps below are
the textbook ones with every free choice fixed):

  draws       every random number is bits(seed, stream, index), a counter-based 64-bit hash (below).
  tree t      trains on `sample`: all rows 0..n-1, or with bootstrap n draws with replacement,
              sample[i] = bits(seed, 2t, i) mod n.
  nodes       numbered in the order they are created, depth first, left subtree before right (so children always
              have a larger number than their parent).  Node `me` holds the multiset `idx` of sample rows.
  leaf when   depth = max_depth (max_depth < 0: no limit), or one class only, or |idx| < min_samples_split,
              or |idx| < 2 * min_samples_leaf, or no admissible cut exists.
  features    with max_features >= F all features are tried in index order.  Otherwise the features are tried in a
              random order (Fisher-Yates: for k = 0..F-2 swap position k with k + bits(seed, 2t+1, 16*me + k) mod (F-k))
              and the search stops once max_features of them have been tried and an admissible cut is known.
  cuts        for feature f sort idx by value; a cut between neighbours a < b (distinct values only) is admissible
              when both sides keep >= min_samples_leaf rows.  Threshold = (a + b) / 2, or a when that rounds to b.
              Rows with value <= threshold go left.
  criterion   gini: minimise  n_l * gini_l + n_r * gini_r  = n - (S_l / n_l + S_r / n_r),  S = sum of squared class
              counts: compared as exact fractions.  entropy: minimise  E_l + E_r,  E = sum_c cnt_c * (ln tot - ln cnt_c)
              in doubles, classes in ascending order, left side first.
  ties        equal cost: lower feature index, then lower threshold.
  leaf class  most frequent class of idx, ties to the lowest id.
  forest      trees t = 0 .. n_estimators-1; prediction = class with most tree votes, ties to the lowest id
              (Section VI-A).
"""
from __future__ import annotations

import math
from dataclasses import dataclass

N_CLASSES = 6
_M64 = (1 << 64) - 1


def _mix(z: int) -> int:
    z = (z + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def bits(seed: int, stream: int, idx: int) -> int:
    key = _mix(_mix(seed & _M64) ^ (stream & _M64))
    return _mix(_mix((idx & _M64) ^ key))


@dataclass
class Opts:
    n_estimators: int = 1
    bootstrap: bool = False
    max_depth: int = -1
    min_samples_leaf: int = 1
    min_samples_split: int = 2
    max_features: int = 10
    criterion: str = "gini"
    seed: int = 0


def _counts(y, rows):
    c = [0] * N_CLASSES
    for i in rows:
        c[y[i]] += 1
    return c


def _entropy_cost(c):
    tot = sum(c)
    e = 0.0
    for k in c:
        if k > 0:
            e += k * (math.log(tot) - math.log(k))
    return e


def best_cut(X, y, idx, f, min_leaf, criterion):
    """Best admissible cut of feature f over the rows idx -> (key, f, threshold) or None; smaller key = better."""
    rows = sorted(idx, key=lambda i: X[i][f])
    n = len(rows)
    total = _counts(y, rows)
    left = [0] * N_CLASSES
    best = None
    for p in range(n - 1):
        left[y[rows[p]]] += 1
        a, b = X[rows[p]][f], X[rows[p + 1]][f]
        nl, nr = p + 1, n - p - 1
        if not (a < b) or nl < min_leaf or nr < min_leaf:
            continue
        right = [t - l for t, l in zip(total, left)]
        if criterion == "gini":
            sl, sr = sum(k * k for k in left), sum(k * k for k in right)
            key = (-(sl * nr + sr * nl), nl * nr)          # fraction num / den, to be minimised
        else:
            key = (_entropy_cost(left) + _entropy_cost(right), 1)
        if best is None or _less(key, best[0]):
            thr = (a + b) / 2
            if thr >= b:
                thr = a
            best = (key, f, thr)
    return best


def _less(k1, k2):
    """k1 < k2 for keys (num, den) with den > 0: exact for integers, plain doubles for entropy (den = 1)."""
    return k1[0] * k2[1] < k2[0] * k1[1]


def _better(c1, c2):
    if _less(c1[0], c2[0]):
        return True
    if _less(c2[0], c1[0]):
        return False
    return (c1[1], c1[2]) < (c2[1], c2[2])


def feature_order(seed, tree_id, node, F, max_features):
    order = list(range(F))
    if max_features >= F:
        return order
    for k in range(F - 1):
        j = k + bits(seed, 2 * tree_id + 1, 16 * node + k) % (F - k)
        order[k], order[j] = order[j], order[k]
    return order


def fit_tree(X, y, o: Opts, tree_id: int = 0) -> dict:
    """X: n rows of F floats (lists or an array), y: n class ids -> tree in the model-file layout."""
    X = [[float(v) for v in row] for row in X]
    y = [int(c) for c in y]
    n, F = len(X), len(X[0])
    sample = [bits(o.seed, 2 * tree_id, i) % n for i in range(n)] if o.bootstrap else list(range(n))
    feature, threshold, left, right, klass = [], [], [], [], []

    def grow(idx, depth):
        me = len(feature)
        c = _counts(y, idx)
        feature.append(-1); threshold.append(0.0); left.append(-1); right.append(-1); klass.append(c.index(max(c)))
        if (o.max_depth >= 0 and depth >= o.max_depth) or sum(1 for k in c if k) <= 1:
            return me
        if len(idx) < o.min_samples_split or len(idx) < 2 * o.min_samples_leaf:
            return me
        best, tried = None, 0
        for f in feature_order(o.seed, tree_id, me, F, o.max_features):
            cand = best_cut(X, y, idx, f, o.min_samples_leaf, o.criterion)
            tried += 1
            if cand is not None and (best is None or _better(cand, best)):
                best = cand
            if tried >= o.max_features and best is not None:
                break
        if best is None:
            return me
        _, f, thr = best
        feature[me], threshold[me], klass[me] = f, thr, -1
        left[me] = grow([i for i in idx if X[i][f] <= thr], depth + 1)
        right[me] = grow([i for i in idx if not X[i][f] <= thr], depth + 1)
        return me

    grow(sample, 0)
    return dict(feature=feature, threshold=threshold, left=left, right=right, klass=klass)


def fit_forest(X, y, o: Opts) -> list:
    return [fit_tree(X, y, o, t) for t in range(o.n_estimators)]


def predict_tree(tree: dict, x) -> int:
    node = 0
    while tree["feature"][node] >= 0:
        node = tree["left"][node] if x[tree["feature"][node]] <= tree["threshold"][node] else tree["right"][node]
    return tree["klass"][node]


def predict(trees: list, X) -> list:
    out = []
    for x in X:
        votes = [0] * N_CLASSES
        for t in trees:
            votes[predict_tree(t, x)] += 1
        out.append(votes.index(max(votes)))
    return out
