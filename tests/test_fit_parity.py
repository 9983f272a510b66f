"""The library's host trainer (mo_model_fit) against the training oracle, node by node and bit for bit, over the
hyper-parameters of Table III; plus its error paths, save / load round trip and batch prediction."""
import itertools

import numpy as np
import pytest

from oracle import cart
from paper_2303_05098_amd import mo, synth
from tests.test_oracle_cart import data


def lib_trees(X, y, tmp_path, **kw):
    mdl = mo.mo_model_fit(X, y, **kw)
    p = str(tmp_path / "m.bin")
    mo.mo_model_save(mdl, p)
    return mdl, mo.read_model(p)


def same(trees_lib, trees_orc):
    assert len(trees_lib) == len(trees_orc)
    for a, b in zip(trees_lib, trees_orc):
        for key in ("feature", "left", "right", "klass"):
            assert a[key] == b[key], key
        assert np.asarray(a["threshold"]).tobytes() == np.asarray(b["threshold"], dtype=np.float64).tobytes()


GRID = [dict(n_estimators=1, bootstrap=0, max_depth=-1, min_samples_leaf=1, min_samples_split=2, max_features=10, criterion="gini"),
        dict(n_estimators=1, bootstrap=0, max_depth=6, min_samples_leaf=1, min_samples_split=2, max_features=10, criterion="entropy"),
        dict(n_estimators=4, bootstrap=1, max_depth=-1, min_samples_leaf=1, min_samples_split=2, max_features=10, criterion="gini"),
        dict(n_estimators=3, bootstrap=1, max_depth=12, min_samples_leaf=3, min_samples_split=10, max_features=4, criterion="entropy"),
        dict(n_estimators=3, bootstrap=0, max_depth=-1, min_samples_leaf=2, min_samples_split=5, max_features=1, criterion="gini"),
        dict(n_estimators=2, bootstrap=1, max_depth=0, min_samples_leaf=1, min_samples_split=2, max_features=9, criterion="gini"),
        dict(n_estimators=2, bootstrap=1, max_depth=3, min_samples_leaf=40, min_samples_split=2, max_features=6, criterion="entropy")]


@pytest.mark.parametrize("kw", GRID, ids=[str(i) for i in range(len(GRID))])
@pytest.mark.parametrize("seed", [1, 2])
def test_trainer_equals_oracle(kw, seed, tmp_path):
    X, y = data(20 + seed, 180, noise=0.15)
    if seed == 2:
        X = np.round(X)                          # few distinct values: equal costs and equal neighbours everywhere
    mdl, trees = lib_trees(X, y, tmp_path, seed=seed * 1000 + 7, **kw)
    o = cart.Opts(seed=seed * 1000 + 7, **{**kw, "bootstrap": bool(kw["bootstrap"])})
    want = cart.fit_forest(X, y, o)
    same(trees, want)
    Xt, _ = data(40 + seed, 150)
    assert mo.mo_predict(mdl, Xt).tolist() == cart.predict(want, Xt)
    assert [mo.mo_select(mdl, x) for x in Xt[:20]] == cart.predict(want, Xt[:20])
    assert mdl.info() == (len(want), sum(len(t["feature"]) for t in want))


def test_sweep_shaped_features():
    """Features with the ranges of real records: sizes up to 1e13 next to densities of 1e-7."""
    n = 160
    u = synth.uniform01(5, 0, np.arange(n * 10)).reshape(n, 10)
    X = np.column_stack([np.floor(10 ** (3 + 4 * u[:, 0]))] * 2 + [np.floor(10 ** (4 + 4 * u[:, 2])), 1 + 30 * u[:, 3], 10 ** (-7 + 5 * u[:, 4]),
                         np.floor(1 + 100 * u[:, 5]), np.floor(5 * u[:, 6]), 20 * u[:, 7], np.floor(10 ** (6 * u[:, 8])), np.floor(12 * u[:, 9])])
    y = (np.floor(u[:, 9] * 3) + 2 * (X[:, 3] > 15)).astype(int) % 6
    for crit in ("gini", "entropy"):
        mdl = mo.mo_model_fit(X, y, n_estimators=5, max_features=3, criterion=crit, seed=3)
        want = cart.fit_forest(X, y, cart.Opts(n_estimators=5, bootstrap=True, max_features=3, criterion=crit, seed=3))
        assert mo.mo_predict(mdl, X).tolist() == cart.predict(want, X)
        assert mdl.info()[1] == sum(len(t["feature"]) for t in want)


def test_defaults_are_the_baseline_column():
    o = mo.fit_opts()
    assert (o.n_estimators, o.bootstrap, o.max_depth, o.min_samples_leaf, o.min_samples_split, o.max_features, o.criterion, o.seed) == \
        (100, 1, -1, 1, 2, 10, mo.MO_GINI, 0)


def test_errors_and_edges(tmp_path):
    X, y = data(3, 30)
    for bad in (dict(n_estimators=0), dict(min_samples_leaf=0), dict(min_samples_split=1), dict(max_features=0),
                dict(max_features=11), dict(criterion=2), dict(bootstrap=2)):
        with pytest.raises(mo.MoError) as e:
            mo.mo_model_fit(X, y, **bad)
        assert e.value.status == mo.MO_E_PARAM
    with pytest.raises(mo.MoError) as e:
        mo.mo_model_fit(X, np.full(30, 6))
    assert e.value.status == mo.MO_E_PARAM
    Xn = X.copy()
    Xn[3, 4] = np.nan
    with pytest.raises(mo.MoError) as e:
        mo.mo_model_fit(Xn, y)
    assert e.value.status == mo.MO_E_PARAM
    with pytest.raises(mo.MoError) as e:
        mo.mo_model_fit(np.zeros((0, 10)), np.zeros(0))
    assert e.value.status == mo.MO_E_SHAPE
    # one sample, and constant features: a single leaf
    m1 = mo.mo_model_fit(X[:1], y[:1], n_estimators=1, bootstrap=0)
    assert m1.info() == (1, 1) and mo.mo_predict(m1, X[:5]).tolist() == [int(y[0])] * 5
    mc = mo.mo_model_fit(np.zeros((6, 10)), [5, 2, 2, 5, 1, 1], n_estimators=1, bootstrap=0)
    assert mc.info() == (1, 1) and mo.mo_select(mc, np.zeros(10)) == 1
    # unwritable path
    with pytest.raises(mo.MoError) as e:
        mo.mo_model_save(m1, str(tmp_path / "no_such_dir" / "m.bin"))
    assert e.value.status == mo.MO_E_MODEL
    # save -> load -> save is the identity, and the loaded model predicts the same
    mdl = mo.mo_model_fit(X, y, n_estimators=3, max_features=3, seed=9)
    p1, p2 = str(tmp_path / "a.bin"), str(tmp_path / "b.bin")
    mo.mo_model_save(mdl, p1)
    back = mo.mo_model_load(p1)
    mo.mo_model_save(back, p2)
    assert open(p1, "rb").read() == open(p2, "rb").read()
    assert np.array_equal(mo.mo_predict(back, X), mo.mo_predict(mdl, X))
    mo.write_model(p2, mo.read_model(p1))
    assert open(p1, "rb").read() == open(p2, "rb").read()
    assert mo.mo_predict(mdl, np.zeros((0, 10))).shape == (0,)
