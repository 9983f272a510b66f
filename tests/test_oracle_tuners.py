"""Pins for tree/forest evaluation and the run-first pick — CPU only."""
import numpy as np
import pytest

from oracle import ref
from paper_2303_05098_amd import synth


def leaf(c):
    return (-1, 0.0, -1, -1, c)


def pack(trees):
    off, f, t, l, r, k = [0], [], [], [], [], []
    for nodes in trees:
        for a in nodes:
            f.append(a[0]); t.append(a[1]); l.append(a[2]); r.append(a[3]); k.append(a[4])
        off.append(len(f))
    return dict(tree_off=off, feature=f, threshold=t, left=l, right=r, klass=k, n_classes=6)


def test_hand_built_tree():
    # x[3] <= 5 ? (x[8] <= 2 ? DIA : CSR) : HYB
    tree = [(3, 5.0, 1, 4, -1), (8, 2.0, 2, 3, -1), leaf(2), leaf(1), leaf(4)]
    mdl = pack([tree])
    x = np.zeros(10)
    x[3], x[8] = 5.0, 2.0
    assert ref.select(mdl, x) == 2          # equality goes left at both nodes
    x[8] = 2.0000001
    assert ref.select(mdl, x) == 1
    x[3] = 5.0000001
    assert ref.select(mdl, x) == 4


def test_majority_vote_and_ties():
    t_coo, t_csr, t_hdc = [leaf(0)], [leaf(1)], [leaf(5)]
    x = np.zeros(10)
    assert ref.select(pack([t_csr, t_hdc, t_hdc]), x) == 5
    assert ref.select(pack([t_hdc, t_csr]), x) == 1         # tie -> lowest id
    assert ref.select(pack([t_hdc, t_csr, t_coo]), x) == 0
    assert ref.select(pack([t_hdc]), x) == 5


def test_malformed_models_are_rejected():
    x = np.zeros(10)
    assert ref.select(pack([[(0, 1.0, 0, 0, -1)]]), x) == -1            # cycle
    assert ref.select(pack([[(0, 1.0, 1, 7, -1), leaf(1)]]), np.ones(10) * 2) == -1   # child out of range
    assert ref.select(pack([[leaf(9)]]), x) == -1                        # class out of range


def test_against_sklearn_trees():
    from sklearn.ensemble import RandomForestClassifier
    from sklearn.tree import DecisionTreeClassifier
    X = synth.uniform_pm1(5, 0, np.arange(400 * 10)).reshape(400, 10) * 10
    y = ((X[:, 0] > 0).astype(int) + 2 * (X[:, 3] > 1) + (X[:, 7] * X[:, 2] > 3)) % 6

    def export(est):
        t = est.tree_
        nodes = []
        for i in range(t.node_count):
            if t.children_left[i] < 0:
                nodes.append((-1, 0.0, -1, -1, int(est.classes_[np.argmax(t.value[i][0])])))
            else:
                nodes.append((int(t.feature[i]), float(t.threshold[i]), int(t.children_left[i]), int(t.children_right[i]), -1))
        return nodes

    dt = DecisionTreeClassifier(max_depth=6, random_state=0).fit(X, y)
    mdl = pack([export(dt)])
    Xt = synth.uniform_pm1(6, 0, np.arange(300 * 10)).reshape(300, 10) * 10
    # scikit-learn compares float32-cast inputs; feed values that are exact in float32
    Xt = Xt.astype(np.float32).astype(np.float64)
    assert [ref.select(mdl, r) for r in Xt] == list(dt.predict(Xt))
    rf = RandomForestClassifier(n_estimators=7, max_depth=5, random_state=0).fit(X, y)
    mdl = pack([export(e) for e in rf.estimators_])
    # hard vote of the exported trees (the paper's majority rule), computed independently here
    votes = np.stack([rf.classes_[e.predict(Xt).astype(int)] for e in rf.estimators_], axis=0)
    want = [int(np.argmax(np.bincount(votes[:, i].astype(int), minlength=6))) for i in range(Xt.shape[0])]
    assert [ref.select(mdl, r) for r in Xt] == want


@pytest.mark.parametrize("ms,want", [
    ([3.0, 2.0, 5.0, 2.5, 9.0, 4.0], 1),
    ([np.nan, 2.0, 1.0, np.nan, 1.0, 4.0], 2),
    ([np.nan] * 6, -1),
    ([1.0, 1.0, 1.0, 1.0, 1.0, 1.0], 0),
    ([np.nan, np.nan, np.nan, np.nan, np.nan, 0.5], 5),
    ([np.inf, 7.0, np.nan, 7.0, 8.0, 9.0], 1),
])
def test_pick(ms, want):
    assert ref.pick(ms) == want
