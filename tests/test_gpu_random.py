"""GPU parity on a spread of sweep matrices (all five families with their random parameters, 1e3 .. 1e5 rows): features
bit-exact, every feasible format's SpMV and 3-column product within tolerance, conversions element by element, and the
way back to CSR, for matrices nobody tuned the kernels on."""
import numpy as np
import pytest

from oracle import ref
from paper_2303_05098_amd import mo, synth
from tests.gpu_util import TOL, gpu_spmv, try_convert, upload
from tests.test_gpu_parity import check_arrays, oracle_feasible
from tests.test_gpu_spmm import check as check_spmm, gpu_spmm, make_X

pytestmark = pytest.mark.gpu

KS = list(range(5000, 5100))


@pytest.mark.parametrize("k", KS)
def test_sweep_matrix(k):
    fam, m, n, rp, ci, v = synth.sweep_matrix(k, 1e3, 1e5)
    dtype = np.float32 if k % 4 == 3 else np.float64
    v = np.asarray(v, dtype=dtype)
    a = upload(m, n, rp, ci, v, dtype)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v.astype(np.float64))
    f, ints = mo.mo_features(a)
    fo, io = ref.features(m, n, ti, tj)
    assert f.tobytes() == fo.tobytes() and ints == io, fam
    x = synth.make_x(n, k).astype(dtype)
    y_ref, mag = ref.spmv(m, n, ti, tj, ta, x.astype(np.float64))
    X = make_X(n, 3, k).astype(dtype)
    Y_ref, Mag = ref.spmm(m, n, ti, tj, ta, X.astype(np.float64))
    for fmt in range(6):
        h = try_convert(a, fmt)
        assert (h is not None) == oracle_feasible(fmt, m, n, ti, tj), (fam, mo.FORMAT_NAMES[fmt])
        if h is None:
            continue
        check_arrays(fam, h.export(), m, n, ti, tj, ta, None)
        err, zeros_ok = ref.spmv_error(gpu_spmv(h, x, m, dtype), y_ref, mag)
        assert err <= TOL[dtype] and zeros_ok, (fam, mo.FORMAT_NAMES[fmt], err)
        check_spmm(gpu_spmm(h, X, m, dtype), Y_ref, Mag, TOL[dtype], (fam, mo.FORMAT_NAMES[fmt]))
        fh, ih = mo.mo_matrix_features(h)
        assert fh.tobytes() == fo.tobytes() and ih == io, (fam, mo.FORMAT_NAMES[fmt])
        e = mo.mo_switch(h, mo.MO_CSR).export()
        assert np.array_equal(e["csr_row_ptr"], rp) and np.array_equal(e["csr_col"], ci) and e["csr_val"].tobytes() == v.tobytes()
        h.free()
