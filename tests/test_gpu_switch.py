"""GPU parity for switching away from any format (mo_switch) and for features gathered from a handle in
whatever format it holds (mo_matrix_features): bit-exact against the oracle's format -> triplets -> ... path."""
import numpy as np
import pytest

from oracle import ref
from paper_2303_05098_amd import mo, synth
from tests.gpu_util import gpu_spmv, try_convert, upload
from tests.test_gpu_parity import CASES, IDS, check_arrays, oracle_feasible
from tests.test_oracle_inverse import oracle_arrays

pytestmark = pytest.mark.gpu

PARAMS = dict(max_fill=256)


def held_triplets(fmt, m, n, ti, tj, ta):
    """What the oracle says a matrix converted to `fmt` holds (DIA drops exact zeros)."""
    return ref.format_to_triplets(fmt, m, n, oracle_arrays(fmt, m, n, ti, tj, ta))


@pytest.mark.parametrize("case", CASES, ids=IDS)
def test_features_from_any_format(case):
    name, m, n, rp, ci, v = case
    a = upload(m, n, rp, ci, v)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    for fmt in range(6):
        h = try_convert(a, fmt, PARAMS)
        if h is None:
            continue
        hi, hj, _ = held_triplets(fmt, m, n, ti, tj, ta)
        for td in ((1, 2), (1, 16)):
            f, ints = mo.mo_matrix_features(h, dict(td_num=td[0], td_den=td[1]))
            fo, io = ref.features(m, n, hi, hj, td)
            assert f.tobytes() == fo.tobytes(), (mo.FORMAT_NAMES[fmt], f, fo)
            assert ints == io
        h.free()


@pytest.mark.parametrize("case", CASES, ids=IDS)
def test_switch_to_csr_and_on(case):
    name, m, n, rp, ci, v = case
    a = upload(m, n, rp, ci, v)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    x = synth.make_x(n, 6)
    y_ref, mag = ref.spmv(m, n, ti, tj, ta, x)
    for src in range(6):
        h = try_convert(a, src, PARAMS)
        if h is None:
            continue
        hi, hj, ha = held_triplets(src, m, n, ti, tj, ta)
        g = mo.mo_switch(h, mo.MO_CSR)
        e = g.export()
        wrp, wc, wv = ref.to_csr(m, hi, hj, ha)
        assert e["nnz"] == wc.shape[0] and np.array_equal(e["csr_row_ptr"], wrp) and np.array_equal(e["csr_col"], wc)
        assert e["csr_val"].tobytes() == wv.tobytes()
        assert np.array_equal(e["csr_row_ptr"], rp) and np.array_equal(e["csr_col"], ci)    # values here are never 0
        h.free()                                                                            # the new handle owns its arrays
        err, ok = ref.spmv_error(gpu_spmv(g, x, m, np.float64), y_ref, mag)
        assert err <= 1e-13 and ok
        # and on to every other format, straight from the source format
        h = try_convert(a, src, PARAMS)
        for dst in range(6):
            feas = oracle_feasible(dst, m, n, hi, hj, 256)
            try:
                d = mo.mo_switch(h, dst, PARAMS)
            except mo.MoError as ex:
                assert ex.status == mo.MO_E_FILL and not feas
                continue
            assert feas
            check_arrays(name, d.export(), m, n, hi, hj, ha, PARAMS)
            err, ok = ref.spmv_error(gpu_spmv(d, x, m, np.float64), y_ref, mag)
            assert err <= 1e-13 and ok, (mo.FORMAT_NAMES[src], mo.FORMAT_NAMES[dst])
            d.free()
        h.free()
        g.free()


def test_stored_zeros():
    """ELL, COO, HYB and the CSR part of HDC keep stored zeros; a DIA slab cannot, and the oracle says the same."""
    m, n, rp, ci, v = synth.random_csr(60, 45, 0.2, 31, 0.1)
    v = v.copy()
    v[::3] = 0.0
    a = upload(m, n, rp, ci, v)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    for fmt in range(6):
        h = mo.mo_convert(a, fmt, PARAMS)
        hi, hj, ha = held_triplets(fmt, m, n, ti, tj, ta)
        e = mo.mo_switch(h, mo.MO_CSR).export()
        wrp, wc, wv = ref.to_csr(m, hi, hj, ha)
        assert np.array_equal(e["csr_row_ptr"], wrp) and np.array_equal(e["csr_col"], wc) and e["csr_val"].tobytes() == wv.tobytes()
        f, ints = mo.mo_matrix_features(h)
        fo, io = ref.features(m, n, hi, hj)
        assert f.tobytes() == fo.tobytes() and ints == io
        if fmt in (mo.MO_COO, mo.MO_CSR, mo.MO_ELL, mo.MO_HYB):
            assert e["nnz"] == rp[-1]
        if fmt == mo.MO_DIA:
            assert e["nnz"] == np.count_nonzero(v)
        h.free()


@pytest.mark.parametrize("dtype", [np.float32])
def test_switch_fp32(dtype):
    m, n, rp, ci, v = synth.config(4, 1 / 128)
    a = upload(m, n, rp, ci, v, dtype)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, np.asarray(v, dtype=dtype).astype(np.float64))
    h = mo.mo_convert(a, mo.MO_HDC)
    d = mo.mo_switch(h, mo.MO_HYB)
    check_arrays("c4", d.export(), m, n, ti, tj, ta, None)
    f, _ = mo.mo_matrix_features(d)
    assert f.tobytes() == ref.features(m, n, ti, tj)[0].tobytes()
