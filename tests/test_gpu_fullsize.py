"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Features and SpMV are compared with the oracle over the whole matrix (the C oracle needs a second or two at
these sizes).  Every exported array of every feasible conversion is compared with the oracle's, byte for byte over
its logical extent, padding included (a few seconds of oracle time per format); before that, as a fast pre-check
that names the broken rule when something is off, (i) a seeded sample of stored entries is looked up where the
definition of each format puts it and (ii) properties that hold at any size are checked (non-padding slots = nnz,
offsets ascending, parts disjoint and complete, closed-form offsets and widths where they exist).  The last test
of each configuration runs the whole online stage (Section III-B): features -> model -> conversion -> SpMV on the
library side against features -> model -> SpMV on the oracle side."""
import os

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2303_05098_amd import mo, synth
from tests.gpu_util import TOL, gpu_spmv, oracle_inputs, try_convert, upload
from tests.test_oracle_features import stencil27_closed_form

pytestmark = pytest.mark.gpu

N_SAMPLE = 20000


def sample_entries(rp, ci, v, seed):
    nnz = int(rp[-1])
    p = np.unique((synth.uniform01(seed, 77, np.arange(N_SAMPLE)) * nnz).astype(np.int64))
    p = np.concatenate([p, [0, nnz - 1]])
    rows = np.searchsorted(rp, p, side="right") - 1
    return p, rows.astype(np.int64), ci[p].astype(np.int64), v[p]


def check_sampled(e, rp, ci, v, dtype, seed, m, n):
    """Every sampled stored entry sits where the format definition puts it."""
    p, i, j, a = sample_entries(rp, ci, v, seed)
    a = a.astype(dtype)
    s = p - rp[i]                                   # position inside its row
    fmt = e["fmt"]
    if fmt == mo.MO_COO:
        assert np.array_equal(e["coo_row"][p], i) and np.array_equal(e["coo_col"][p], j) and np.array_equal(e["coo_val"][p], a)
        assert e["nnz_coo"] == rp[-1]
        assert np.all(np.diff(e["coo_row"].astype(np.int64) * n + e["coo_col"]) > 0)      # (row, col) strictly ascending
    if fmt == mo.MO_DIA:
        k = np.searchsorted(e["dia_off"], j - i)
        assert np.array_equal(e["dia_off"][k], j - i)
        assert np.array_equal(e["dia_val"][k, i], a)
        assert np.all(np.diff(e["dia_off"]) > 0)
    if fmt == mo.MO_ELL:
        assert np.array_equal(e["ell_col"][s, i], j) and np.array_equal(e["ell_val"][s, i], a)
        assert int((e["ell_col"][:, :m] >= 0).sum()) == rp[-1]
        lens = np.diff(rp)
        assert e["k"] == lens.max()
        # rows are packed from slot 0: the number of non-padding slots of a row is its length, padding values are +0
        assert np.array_equal((e["ell_col"][:, :m] >= 0).sum(axis=0), lens)
        assert not np.any(e["ell_val"][:, :m][e["ell_col"][:, :m] < 0])
    if fmt == mo.MO_HYB:
        K = e["k"]
        in_ell = s < K
        assert np.array_equal(e["ell_col"][s[in_ell], i[in_ell]], j[in_ell])
        assert np.array_equal(e["ell_val"][s[in_ell], i[in_ell]], a[in_ell])
        lens = np.diff(rp).astype(np.int64)
        surplus = np.maximum(lens - K, 0)
        cptr = np.concatenate([[0], np.cumsum(surplus)])
        assert e["nnz_coo"] == cptr[-1]
        q = cptr[i[~in_ell]] + (s[~in_ell] - K)
        assert np.array_equal(e["coo_row"][q], i[~in_ell]) and np.array_equal(e["coo_col"][q], j[~in_ell])
        assert np.array_equal(e["coo_val"][q], a[~in_ell])
        assert int((e["ell_col"][:, :m] >= 0).sum()) + e["nnz_coo"] == rp[-1]
        # K_H by its definition: largest k with #{len >= k} * 3 >= m
        ok = [k for k in range(int(lens.max()) + 1) if int((lens >= k).sum()) * 3 >= m]
        assert K == max(ok)
    if fmt == mo.MO_HDC:
        d = j - i
        k = np.searchsorted(e["dia_off"], d)
        k = np.minimum(k, max(e["nd"] - 1, 0))
        on_dia = (e["dia_off"][k] == d) if e["nd"] else np.zeros(d.shape, bool)
        assert np.array_equal(e["dia_val"][k[on_dia], i[on_dia]], a[on_dia])
        crp = e["csr_row_ptr"].astype(np.int64)
        assert crp[0] == 0 and crp[-1] == e["nnz_csr"] and np.all(np.diff(crp) >= 0)
        for ii, jj, aa in zip(i[~on_dia], j[~on_dia], a[~on_dia]):
            seg = e["csr_col"][crp[ii]:crp[ii + 1]]
            pos = np.searchsorted(seg, jj)
            assert seg[pos] == jj and e["csr_val"][crp[ii] + pos] == aa
        # parts complete: entries on kept diagonals + remainder = nnz
        cnt = np.bincount((ci.astype(np.int64) - np.repeat(np.arange(m, dtype=np.int64), np.diff(rp))) + (m - 1), minlength=m + n - 1)
        kept = cnt[e["dia_off"].astype(np.int64) + (m - 1)].sum() if e["nd"] else 0
        assert kept + e["nnz_csr"] == rp[-1]
        true = np.nonzero((cnt >= 1) & (cnt * 2 >= min(m, n)))[0] - (m - 1)
        assert np.array_equal(e["dia_off"], true)


def same_bytes(got, want, what):
    """Equal as bit patterns (so that -0.0 in place of +0.0 padding, or a NaN, cannot pass as equal)."""
    got, want = np.ascontiguousarray(got), np.ascontiguousarray(want)
    assert got.dtype == want.dtype and got.shape == want.shape, (what, got.dtype, want.dtype, got.shape, want.shape)
    u = {4: np.uint32, 8: np.uint64}[got.dtype.itemsize]
    if not np.array_equal(got.view(u), want.view(u)):
        bad = np.nonzero(got.view(u).reshape(-1) != want.view(u).reshape(-1))[0]
        raise AssertionError(f"{what}: {bad.size} of {got.size} elements differ, first at flat index {int(bad[0])}: "
                             f"{got.reshape(-1)[bad[0]]!r} != {want.reshape(-1)[bad[0]]!r}")


def check_full(e, m, n, ti, tj, ta, dtype):
    """Every exported array against the oracle's conversion of the same triplets, over the logical extent [:, :m]."""
    fmt = e["fmt"]
    cast = lambda a: a.astype(dtype)   # noqa: E731  (exact: the triplets hold dtype values promoted to fp64)
    if fmt == mo.MO_COO:
        row, col, val = ref.to_coo(ti, tj, ta)
        assert e["nnz_coo"] == row.shape[0]
        same_bytes(e["coo_row"], row, "coo_row"); same_bytes(e["coo_col"], col, "coo_col"); same_bytes(e["coo_val"], cast(val), "coo_val")
    elif fmt == mo.MO_DIA:
        off, val = ref.to_dia(m, n, ti, tj, ta)
        assert e["nd"] == off.shape[0]
        same_bytes(e["dia_off"], off, "dia_off"); same_bytes(e["dia_val"][:, :m], cast(val), "dia_val")
    elif fmt == mo.MO_ELL:
        k, col, val = ref.to_ell(m, ti, tj, ta)
        assert e["k"] == k
        same_bytes(e["ell_col"][:, :m], col, "ell_col"); same_bytes(e["ell_val"][:, :m], cast(val), "ell_val")
    elif fmt == mo.MO_HYB:
        o = ref.to_hyb(m, ti, tj, ta)
        assert e["k"] == o["k"] and e["nnz_coo"] == o["coo_row"].shape[0]
        same_bytes(e["ell_col"][:, :m], o["ell_col"], "hyb ell_col"); same_bytes(e["ell_val"][:, :m], cast(o["ell_val"]), "hyb ell_val")
        same_bytes(e["coo_row"], o["coo_row"], "hyb coo_row"); same_bytes(e["coo_col"], o["coo_col"], "hyb coo_col")
        same_bytes(e["coo_val"], cast(o["coo_val"]), "hyb coo_val")
    elif fmt == mo.MO_HDC:
        o = ref.to_hdc(m, n, ti, tj, ta)
        assert e["nd"] == o["dia_off"].shape[0] and e["nnz_csr"] == o["csr_col"].shape[0]
        same_bytes(e["dia_off"], o["dia_off"], "hdc dia_off"); same_bytes(e["dia_val"][:, :m], cast(o["dia_val"]), "hdc dia_val")
        same_bytes(e["csr_row_ptr"], o["csr_row_ptr"], "hdc row_ptr"); same_bytes(e["csr_col"], o["csr_col"], "hdc csr_col")
        same_bytes(e["csr_val"], cast(o["csr_val"]), "hdc csr_val")


def oracle_model(path):
    """The committed model file, parsed on the Python side, in the form the oracle's forest walk takes."""
    trees = mo.read_model(path)
    cat = {k: [] for k in ("feature", "threshold", "left", "right", "klass")}
    off = [0]
    for t in trees:
        for k in cat:
            cat[k] += list(t[k])
        off.append(len(cat["feature"]))
    return dict(tree_off=off, n_classes=6, **cat)


MODEL_PATH = os.path.join(os.path.dirname(os.path.abspath(mo.__file__)), "models", "mi355x_forest.bin")


def run_chain(c, dtype):
    """Online stage, library against oracle: the format the committed model names for the library's features must be
    the one the oracle's forest walk names for the oracle's features; the matrix converted to it must multiply right."""
    m, n, rp, ci, v = synth.config(c)
    v = np.asarray(v, dtype=dtype)
    a = upload(m, n, rp, ci, v, dtype)
    x = synth.make_x(n, synth.BASE_SEED + c)
    ti, tj, ta, xo = oracle_inputs(rp, ci, v, x, dtype)
    f, _ = mo.mo_features(a)
    fo, _ = ref.features(m, n, ti, tj)
    assert f.tobytes() == fo.tobytes()
    mdl = mo.mo_model_load(MODEL_PATH)
    fmt = mo.mo_select(mdl, f)
    assert fmt == ref.select(oracle_model(MODEL_PATH), fo)
    h = try_convert(a, fmt)
    assert h is not None, f"the model names {mo.FORMAT_NAMES[fmt]}, which is not feasible on config {c}"
    y_ref, mag = ref.spmv(m, n, ti, tj, ta, xo)
    err, zeros_ok = ref.spmv_error(gpu_spmv(h, x, m, dtype), y_ref, mag)
    assert err <= TOL[dtype] and zeros_ok, (mo.FORMAT_NAMES[fmt], err)
    h.free()
    mdl.free()


def run_config(c, dtype, expect_infeasible=()):
    m, n, rp, ci, v = synth.config(c)
    v = np.asarray(v, dtype=dtype)
    a = upload(m, n, rp, ci, v, dtype)
    x = synth.make_x(n, synth.BASE_SEED + c)
    ti, tj, ta, xo = oracle_inputs(rp, ci, v, x, dtype)
    y_ref, mag = ref.spmv(m, n, ti, tj, ta, xo)
    f, ints = mo.mo_features(a)
    fo, io = ref.features(m, n, ti, tj)
    assert f.tobytes() == fo.tobytes() and ints == io
    # the second operation at full size: 8 right-hand sides, every entry of Y against the oracle
    K = 8
    X = synth.uniform_pm1(synth.BASE_SEED + 40 + c, 0, np.arange(n * K)).reshape(n, K).astype(dtype)
    Y_ref, Mag = ref.spmm(m, n, ti, tj, ta, X.astype(np.float64))
    Xd = torch.as_tensor(X).cuda()
    for fmt in range(6):
        h = try_convert(a, fmt)
        if mo.FORMAT_NAMES[fmt] in expect_infeasible:
            assert h is None
            continue
        assert h is not None
        Yd = torch.full((m, K), float("nan"), dtype=Xd.dtype, device="cuda")
        mo.mo_spmm(h, Xd, Yd)
        torch.cuda.synchronize()
        Y = Yd.cpu().numpy().astype(np.float64)
        nz = Mag > 0
        assert float(np.max(np.abs(Y[nz] - Y_ref[nz]) / Mag[nz])) <= TOL[dtype], mo.FORMAT_NAMES[fmt]
        assert np.all(Y[~nz] == 0)
        del Yd, Y
        y = gpu_spmv(h, x, m, dtype)
        err, zeros_ok = ref.spmv_error(y, y_ref, mag)
        assert err <= TOL[dtype] and zeros_ok, (mo.FORMAT_NAMES[fmt], err)
        assert gpu_spmv(h, x, m, dtype).tobytes() == y.tobytes()
        if fmt != mo.MO_CSR:
            e = h.export()
            check_sampled(e, rp, ci, v, dtype, 100 + c, m, n)
            check_full(e, m, n, ti, tj, ta, dtype)
            del e
        # features gathered from the held format, and the way back to CSR: no value of these inputs is 0, so both
        # must reproduce what the CSR input gives, bit for bit
        assert np.count_nonzero(v) == rp[-1]
        fh, ih = mo.mo_matrix_features(h)
        assert fh.tobytes() == fo.tobytes() and ih == io, mo.FORMAT_NAMES[fmt]
        if fmt != mo.MO_CSR:
            g = mo.mo_switch(h, mo.MO_CSR)
            e = g.export()
            assert np.array_equal(e["csr_row_ptr"], rp) and np.array_equal(e["csr_col"], ci)
            assert e["csr_val"].tobytes() == v.tobytes(), mo.FORMAT_NAMES[fmt]
            del e
            g.free()
        h.free()
        torch.cuda.empty_cache()
    return f, ints


def test_c2_stencil27_128():
    f, ints = run_config(2, np.float64)
    counts, nnz, sumsq, diag = stencil27_closed_form(128)
    assert ints["nnz"] == nnz and ints["sum_sq_row"] == sumsq and ints["n_diag"] == 27 and ints["n_true_diag"] == 27
    assert ints["max_row"] == 27 and ints["min_row"] == 8


def test_c3_lognormal():
    run_config(3, np.float64, expect_infeasible=("DIA", "ELL"))


@pytest.mark.parametrize("dtype", [np.float64, np.float32], ids=["f64", "f32"])
def test_c4_banded_scatter(dtype):
    f, ints = run_config(4, dtype, expect_infeasible=("DIA",))
    assert ints["nnz"] == 38903548 and ints["n_true_diag"] == 9


@pytest.mark.parametrize("c,dtype", [(1, np.float64), (2, np.float64), (3, np.float64), (4, np.float64), (4, np.float32)],
                         ids=["c1", "c2", "c3", "c4-f64", "c4-f32"])
def test_online_stage_chain(c, dtype):
    run_chain(c, dtype)
