"""Host-side tree training: pinned against scikit-learn (test-only) and hand-computable cases."""
import numpy as np
import pytest

from paper_2303_05098_amd import fit, synth


def data(seed, n=300):
    X = synth.uniform_pm1(seed, 0, np.arange(n * 10)).reshape(n, 10) * 10
    y = ((X[:, 0] > 0).astype(int) + 2 * (X[:, 3] > 1) + (X[:, 7] + X[:, 2] > 3)) % 6
    return X, y


@pytest.mark.parametrize("seed,depth", [(1, 3), (2, 6), (3, 12)])
def test_matches_sklearn_cart(seed, depth):
    from sklearn.tree import DecisionTreeClassifier
    X, y = data(seed)
    t = fit.fit_tree(X, y, max_depth=depth)
    sk = DecisionTreeClassifier(criterion="gini", max_depth=depth, random_state=0).fit(X, y)
    # Both are greedy gini trees with midpoint thresholds, so they agree on the training set.  Small nodes can have
    # several splits of equal gain (scikit-learn picks among them by a random feature order, this code by lowest
    # feature index), so fresh points may differ on a few per cent of the samples.
    Xt, _ = data(seed + 50, 500)
    assert np.array_equal(fit.predict_tree(t, X), sk.predict(X))
    assert np.mean(fit.predict_tree(t, Xt) == sk.predict(Xt)) >= 0.95


def test_hand_case_and_tie_rules():
    # one feature separates perfectly at 0.5 -> root split on feature 0 (lowest index wins the tie with feature 1)
    X = np.zeros((8, 10))
    X[:, 0] = [0, 0, 0, 0, 1, 1, 1, 1]
    X[:, 1] = X[:, 0]
    y = np.array([1, 1, 1, 1, 4, 4, 4, 4])
    t = fit.fit_tree(X, y, max_depth=3)
    assert t["feature"] == [0, -1, -1] and t["threshold"][0] == 0.5 and t["klass"] == [-1, 1, 4]
    assert t["left"][0] == 1 and t["right"][0] == 2
    # constant features -> a single leaf with the majority class, ties to the lowest id
    t = fit.fit_tree(np.zeros((4, 10)), np.array([5, 2, 2, 5]), max_depth=3)
    assert t["feature"] == [-1] and t["klass"] == [2]
    # depth limit
    X, y = data(4)
    t = fit.fit_tree(X, y, max_depth=2)
    assert len(t["feature"]) <= 7


def test_children_follow_parents():
    X, y = data(5)
    t = fit.fit_tree(X, y, max_depth=8)
    for i, f in enumerate(t["feature"]):
        if f >= 0:
            assert t["left"][i] > i and t["right"][i] > i


def test_stratified_folds_and_metrics():
    y = np.array([1] * 50 + [2] * 10 + [5] * 5)
    fold = fit.stratified_folds(y, 5)
    for c, n in ((1, 50), (2, 10), (5, 5)):
        cnt = np.bincount(fold[y == c], minlength=5)
        assert cnt.sum() == n and cnt.max() - cnt.min() <= 1
    assert np.bincount(fold, minlength=5).max() - np.bincount(fold, minlength=5).min() <= 1
    assert fit.accuracy([1, 1, 2, 5], [1, 2, 2, 5]) == 0.75
    # recalls: class 1 -> 1/2, class 2 -> 1, class 5 -> 1
    assert abs(fit.balanced_accuracy([1, 1, 2, 5], [1, 2, 2, 5]) - (0.5 + 1 + 1) / 3) < 1e-15
    from sklearn.metrics import balanced_accuracy_score
    yt = (synth.uniform01(1, 0, np.arange(200)) * 4).astype(int)
    yp = (synth.uniform01(2, 0, np.arange(200)) * 4).astype(int)
    assert abs(fit.balanced_accuracy(yt, yp) - balanced_accuracy_score(yt, yp)) < 1e-12


def test_cross_validate_runs_and_model_roundtrip(tmp_path):
    from oracle import ref
    from paper_2303_05098_amd import mo
    X, y = data(6, 200)
    cv = fit.cross_validate(X, y, 5, max_depth=6)
    assert 0.5 < cv["accuracy"] <= 1.0 and len(cv["per_fold"]) == 5
    t = fit.fit_tree(X, y, 6)
    p = str(tmp_path / "t.bin")
    mo.write_model(p, [t])
    mdl = mo.mo_model_load(p)
    om = dict(tree_off=[0, len(t["feature"])], n_classes=6, **t)
    for x, want in zip(X, fit.predict_tree(t, X)):
        assert mo.mo_select(mdl, x) == want == ref.select(om, x)
