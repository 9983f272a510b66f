"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Features and SpMV are compared with the oracle over the whole matrix (the C oracle needs a second or two at
these sizes).  The converted arrays are too large to rebuild on the CPU in reasonable time, so they are checked
(i) entry by entry on a seeded sample of stored entries, straight from the definition of each format, and
(ii) through properties that hold at any size (non-padding slots = nnz, offsets ascending, parts disjoint and
complete, closed-form offsets and widths where they exist)."""
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
            check_sampled(h.export(), rp, ci, v, dtype, 100 + c, m, n)
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
