"""The C-ABI library without a GPU: it loads, exports what include/mo.h declares, and its host-only logic
(argument checks, mo_pick, model loading, mo_select) agrees with the oracle."""
import ctypes as C
import os
import re
import struct

import numpy as np
import pytest

from oracle import ref
from paper_2303_05098_amd import mo, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_match_header():
    text = open(os.path.join(ROOT, "include", "mo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(mo_[a-z_]+)\s*\(", text))
    assert declared == set(mo.EXPORTS), declared ^ set(mo.EXPORTS)
    for name in declared:
        assert hasattr(mo.lib, name), name


def test_default_params():
    p = mo.mo_params()
    mo.lib.mo_default_params(C.byref(p))
    assert (p.td_num, p.td_den, p.hyb_num, p.hyb_den, p.max_fill, p.max_slots) == (1, 2, 1, 3, 16, 1 << 62)


def test_strerror_covers_every_status():
    seen = {mo.lib.mo_strerror(s).decode() for s in range(12)}
    assert len(seen) == 12 and "unknown status" not in seen
    assert mo.lib.mo_strerror(12).decode() == "unknown status"


@pytest.mark.parametrize("ms", [
    [3.0, 2.0, 5.0, 2.5, 9.0, 4.0], [np.nan, 2.0, 1.0, np.nan, 1.0, 4.0], [1.0] * 6,
    [np.nan, np.nan, np.nan, np.nan, np.nan, 0.5], [np.inf, 7.0, np.nan, 7.0, 8.0, 9.0],
])
def test_pick_matches_oracle(ms):
    assert mo.mo_pick(ms) == ref.pick(ms)


def test_pick_all_nan_is_an_error():
    with pytest.raises(mo.MoError) as e:
        mo.mo_pick([np.nan] * 6)
    assert e.value.status == mo.MO_E_PARAM
    assert ref.pick([np.nan] * 6) == -1


def test_pick_random_vectors():
    u = synth.uniform01(3, 0, np.arange(600)).reshape(100, 6)
    u[u < 0.2] = np.nan
    u = np.round(u, 1)               # force ties
    for row in u:
        if np.all(np.isnan(row)):
            continue
        assert mo.mo_pick(row) == ref.pick(row)


def random_forest_arrays(seed, n_trees, depth):
    """Random complete-ish trees in the model layout (children after parents)."""
    trees = []
    for t in range(n_trees):
        feature, thr, left, right, klass = [], [], [], [], []
        u = iter(synth.uniform01(seed, t, np.arange(4096)))

        def grow(d):
            i = len(feature)
            feature.append(-1); thr.append(0.0); left.append(-1); right.append(-1); klass.append(int(next(u) * 6))
            if d < depth and next(u) < 0.8:
                feature[i] = int(next(u) * 10)
                thr[i] = round(next(u) * 20 - 10, 1)
                left[i] = grow(d + 1)
                right[i] = grow(d + 1)
                klass[i] = -1
            return i

        grow(0)
        trees.append(dict(feature=feature, threshold=thr, left=left, right=right, klass=klass))
    return trees


def to_oracle_model(trees):
    off = [0]
    cat = {k: [] for k in ("feature", "threshold", "left", "right", "klass")}
    for t in trees:
        for k in cat:
            cat[k] += list(t[k])
        off.append(len(cat["feature"]))
    return dict(tree_off=off, n_classes=6, **cat)


@pytest.mark.parametrize("n_trees,depth", [(1, 5), (7, 4), (20, 6)])
def test_select_matches_oracle(tmp_path, n_trees, depth):
    trees = random_forest_arrays(11 + n_trees, n_trees, depth)
    path = str(tmp_path / "m.bin")
    mo.write_model(path, trees)
    mdl = mo.mo_model_load(path)
    assert mdl.info() == (n_trees, sum(len(t["feature"]) for t in trees))
    om = to_oracle_model(trees)
    X = np.round(synth.uniform_pm1(5, 1, np.arange(300 * 10)).reshape(300, 10) * 10, 1)   # ties with thresholds occur
    for x in X:
        assert mo.mo_select(mdl, x) == ref.select(om, x)
    mdl.free()


def test_model_file_errors(tmp_path):
    good = random_forest_arrays(1, 2, 3)
    path = str(tmp_path / "g.bin")
    mo.write_model(path, good)
    blob = open(path, "rb").read()

    def status_of(data):
        p = str(tmp_path / "x.bin")
        open(p, "wb").write(data)
        try:
            mo.mo_model_load(p).free()
            return mo.MO_OK
        except mo.MoError as e:
            return e.status

    assert status_of(blob) == mo.MO_OK
    assert status_of(blob[:-3]) == mo.MO_E_MODEL                       # truncated
    assert status_of(blob + b"\0") == mo.MO_E_MODEL                    # trailing bytes
    assert status_of(b"XXMDL1\0\0" + blob[8:]) == mo.MO_E_MODEL        # wrong magic
    assert status_of(blob[:8] + struct.pack("<4i", 2, 10, 6, 2) + blob[24:]) == mo.MO_E_MODEL   # version
    assert status_of(blob[:8] + struct.pack("<4i", 1, 9, 6, 2) + blob[24:]) == mo.MO_E_MODEL    # n_features
    assert status_of(blob[:8] + struct.pack("<4i", 1, 10, 6, 0) + blob[24:]) == mo.MO_E_MODEL   # no trees

    def one_tree(feature, thr, left, right, klass):
        return [dict(feature=feature, threshold=thr, left=left, right=right, klass=klass)]

    def st(trees):
        p = str(tmp_path / "y.bin")
        mo.write_model(p, trees)
        try:
            mo.mo_model_load(p).free()
            return mo.MO_OK
        except mo.MoError as e:
            return e.status

    assert st(one_tree([0, -1, -1], [1.0, 0, 0], [1, -1, -1], [2, -1, -1], [-1, 1, 2])) == mo.MO_OK
    assert st(one_tree([10, -1, -1], [1.0, 0, 0], [1, -1, -1], [2, -1, -1], [-1, 1, 2])) == mo.MO_E_MODEL   # feature >= 10
    assert st(one_tree([0, -1, -1], [1.0, 0, 0], [1, -1, -1], [3, -1, -1], [-1, 1, 2])) == mo.MO_E_MODEL    # child out of range
    assert st(one_tree([0, -1, -1], [1.0, 0, 0], [0, -1, -1], [2, -1, -1], [-1, 1, 2])) == mo.MO_E_MODEL    # cycle
    assert st(one_tree([0, -1, -1], [1.0, 0, 0], [1, -1, -1], [2, -1, -1], [-1, 6, 2])) == mo.MO_E_MODEL    # class out of range
    assert st(one_tree([0, -1, -1], [float("nan"), 0, 0], [1, -1, -1], [2, -1, -1], [-1, 1, 2])) == mo.MO_E_MODEL
    with pytest.raises(mo.MoError):
        mo.mo_model_load(str(tmp_path / "does_not_exist.bin"))


def test_argument_checks_need_no_gpu():
    out = (C.c_double * 10)()
    h = C.c_void_p()

    def feat(st, params=None):
        return mo.lib.mo_features(C.byref(st), params, out, None, None)

    dummy = 0x1000
    ok = mo.mo_csr(4, 4, 4, dummy, dummy, dummy, mo.MO_F64)
    assert mo.lib.mo_features(None, None, out, None, None) == mo.MO_E_NULL
    assert mo.lib.mo_features(C.byref(ok), None, None, None, None) == mo.MO_E_NULL
    assert feat(mo.mo_csr(0, 4, 0, dummy, dummy, dummy, mo.MO_F64)) == mo.MO_E_SHAPE
    assert feat(mo.mo_csr(4, 0, 0, dummy, dummy, dummy, mo.MO_F64)) == mo.MO_E_SHAPE
    assert feat(mo.mo_csr(4, 4, -1, dummy, dummy, dummy, mo.MO_F64)) == mo.MO_E_SHAPE
    assert feat(mo.mo_csr(4, 4, 1 << 31, dummy, dummy, dummy, mo.MO_F64)) == mo.MO_E_SHAPE
    assert feat(mo.mo_csr(1 << 30, 1 << 30, 4, dummy, dummy, dummy, mo.MO_F64)) == mo.MO_E_SHAPE
    assert feat(mo.mo_csr(4, 4, 4, None, dummy, dummy, mo.MO_F64)) == mo.MO_E_NULL
    assert feat(mo.mo_csr(4, 4, 4, dummy, None, dummy, mo.MO_F64)) == mo.MO_E_NULL
    assert feat(mo.mo_csr(4, 4, 4, dummy, dummy, None, mo.MO_F64)) == mo.MO_E_NULL
    assert feat(mo.mo_csr(4, 4, 4, dummy, dummy, dummy, 7)) == mo.MO_E_DTYPE
    bad = mo.mo_params(1, 0, 1, 3, 16, 1 << 62)
    assert feat(ok, C.byref(bad)) == mo.MO_E_PARAM
    bad = mo.mo_params(1, 2, -1, 3, 16, 1 << 62)
    assert feat(ok, C.byref(bad)) == mo.MO_E_PARAM
    assert mo.lib.mo_convert(C.byref(ok), 6, None, C.byref(h), None) == mo.MO_E_FORMAT
    assert mo.lib.mo_convert(C.byref(ok), -1, None, C.byref(h), None) == mo.MO_E_FORMAT
    assert mo.lib.mo_convert(C.byref(ok), 1, None, None, None) == mo.MO_E_NULL
    assert mo.lib.mo_spmv(None, dummy, dummy, None) == mo.MO_E_NULL
    assert mo.lib.mo_matrix_export(None, None) == mo.MO_E_NULL
    mo.lib.mo_matrix_free(None)
    mo.lib.mo_model_free(None)
    # the calls added for switching, the second operation, training and files
    assert mo.lib.mo_switch(None, 1, None, C.byref(h), None) == mo.MO_E_NULL
    assert mo.lib.mo_switch(dummy, 1, None, None, None) == mo.MO_E_NULL
    assert mo.lib.mo_matrix_features(None, None, out, None, None) == mo.MO_E_NULL
    assert mo.lib.mo_spmm(None, dummy, dummy, 4, None) == mo.MO_E_NULL
    best, ms6 = C.c_int(-1), (C.c_double * 6)()
    for k in (0, -3, 65):
        assert mo.lib.mo_tune_spmm(C.byref(ok), k, None, None, C.byref(best), ms6, None, None) == mo.MO_E_PARAM
    assert mo.lib.mo_tune_spmm(C.byref(ok), 4, None, None, None, ms6, None, None) == mo.MO_E_NULL
    assert mo.lib.mo_tune(C.byref(ok), None, None, None, ms6, None, None) == mo.MO_E_NULL
    assert mo.lib.mo_model_fit(None, None, 5, None, C.byref(h)) == mo.MO_E_NULL
    assert mo.lib.mo_model_save(None, b"/tmp/x") == mo.MO_E_NULL
    assert mo.lib.mo_predict(None, None, 0, None) == mo.MO_E_NULL
    i64 = C.c_int64()
    assert mo.lib.mo_mtx_read(None, C.byref(i64), C.byref(i64), C.byref(i64), C.byref(h), C.byref(h), C.byref(h)) == mo.MO_E_NULL
    mo.lib.mo_host_free(None)


def test_features_finalize_matches_the_oracle():
    """The host half of mo_features on its own (Table I): from the oracle's integer counts it must give the oracle's
    ten doubles bit for bit, on matrices with empty rows, rectangular shapes and a large closed-form case."""
    cases = [synth.config(1), synth.random_csr(300, 1000, 0.02, 5, 0.3), synth.random_csr(1000, 130, 0.05, 6, 0.1),
             synth.config(3, 1 / 64), synth.config(2, 0.1)]
    for m, n, rp, ci, v in cases:
        ti, tj, _ = ref.csr_to_triplets(rp, ci, v)
        fo, io = ref.features(m, n, ti, tj)
        f = mo.mo_features_finalize(io)
        assert f.tobytes() == fo.tobytes()
    # 128^3 stencil from its closed-form integers (no matrix needed)
    g = 128
    nnz = (3 * g - 2) ** 3
    counts = {27: (g - 2) ** 3, 18: 6 * (g - 2) ** 2, 12: 12 * (g - 2), 8: 8}
    ints = dict(m=g ** 3, n=g ** 3, nnz=nnz, max_row=27, min_row=8, n_diag=27, n_true_diag=27,
                sum_sq_row=sum(k * k * c for k, c in counts.items()))
    f = mo.mo_features_finalize(ints)
    assert f[3] == nnz / g ** 3 and abs(f[7] - 1.9148405) < 1e-6 and f[8] == 27.0
    bad = dict(ints, m=0)
    with pytest.raises(mo.MoError) as e:
        mo.mo_features_finalize(bad)
    assert e.value.status == mo.MO_E_SHAPE
