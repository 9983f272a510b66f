"""GPU parity of the multi-vector product Y = A X (mo_spmm) in every format against the oracle, element by element:
max |Y - Y_ref| / (|A||X|) <= 1e-13 (fp64) / 1e-5 (fp32), entries with (|A||X|) = 0 exactly zero; several widths k
including ones that are not powers of two; run-to-run bit identity; the run-first tuner for this operation."""
import math

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2303_05098_amd import mo, synth
from tests.gpu_util import TOL, try_convert, upload
from tests.test_gpu_parity import CASES, IDS

pytestmark = pytest.mark.gpu

PARAMS = dict(max_fill=256)


def make_X(n, k, seed):
    return synth.uniform_pm1(seed, 40, np.arange(n * k)).reshape(n, k)


def gpu_spmm(h, X, m, dtype):
    x = torch.as_tensor(np.ascontiguousarray(X, dtype=dtype)).cuda()
    y = torch.full((m, X.shape[1]), float("nan"), dtype=x.dtype, device="cuda")
    mo.mo_spmm(h, x, y)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def check(Y, Y_ref, mag, tol, what):
    nz = mag > 0
    err = float(np.max(np.abs(Y.astype(np.float64)[nz] - Y_ref[nz]) / mag[nz])) if nz.any() else 0.0
    assert err <= tol, (what, err)
    assert np.all(Y[~nz] == 0), what


@pytest.mark.parametrize("case", CASES, ids=IDS)
def test_spmm_all_formats(case):
    name, m, n, rp, ci, v = case
    a = upload(m, n, rp, ci, v)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    for k in (1, 3, 8):
        X = make_X(n, k, 50 + k)
        Y_ref, mag = ref.spmm(m, n, ti, tj, ta, X)
        for fmt in range(6):
            h = try_convert(a, fmt, PARAMS)
            if h is None:
                continue
            Y = gpu_spmm(h, X, m, np.float64)
            check(Y, Y_ref, mag, TOL[np.float64], (name, mo.FORMAT_NAMES[fmt], k))
            assert gpu_spmm(h, X, m, np.float64).tobytes() == Y.tobytes()
            h.free()


def test_spmm_fp32_and_wide():
    m, n, rp, ci, v = synth.config(4, 1 / 64)
    for dtype, k in ((np.float32, 5), (np.float64, 64), (np.float32, 32), (np.float64, 2), (np.float32, 4), (np.float64, 16), (np.float64, 32)):
        a = upload(m, n, rp, ci, v, dtype)
        ti, tj, ta = ref.csr_to_triplets(rp, ci, np.asarray(v, dtype=dtype).astype(np.float64))
        X = make_X(n, k, 7).astype(dtype)
        Y_ref, mag = ref.spmm(m, n, ti, tj, ta, X.astype(np.float64))
        for fmt in (mo.MO_COO, mo.MO_CSR, mo.MO_ELL, mo.MO_HYB, mo.MO_HDC):
            h = mo.mo_convert(a, fmt)
            check(gpu_spmm(h, X, m, dtype), Y_ref, mag, TOL[dtype], (mo.FORMAT_NAMES[fmt], dtype, k))
            h.free()


@pytest.mark.parametrize("cname", ["c2s", "c4s", "dense", "band40", "band30s", "very_long_rows", "rect_wide", "rect_tall", "bulge"])
def test_spmm_fp32_pieces(cname):
    """fp32 panels are fetched as 16-byte pieces of four floats whatever the alignment of the rows of X: widths whose rows
    start on 4-, 8- and 16-byte boundaries, on matrices that reach the window kernel, the direct DIA kernel with several
    passes, the fused remainder, long rows and rectangular shapes."""
    name, m, n, rp, ci, v = CASES[IDS.index(cname)]
    a = upload(m, n, rp, ci, v, np.float32)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, np.asarray(v, dtype=np.float32).astype(np.float64))
    for k in (5, 8, 12, 17):
        X = make_X(n, k, 60 + k).astype(np.float32)
        Y_ref, mag = ref.spmm(m, n, ti, tj, ta, X.astype(np.float64))
        for fmt in range(6):
            h = try_convert(a, fmt, PARAMS)
            if h is None:
                continue
            check(gpu_spmm(h, X, m, np.float32), Y_ref, mag, TOL[np.float32], (name, mo.FORMAT_NAMES[fmt], k))
            h.free()


def test_spmm_k1_equals_spmv_layout():
    """k = 1 is SpMV with the same operands."""
    m, n, rp, ci, v = synth.config(2, 0.19)
    a = upload(m, n, rp, ci, v)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    x = synth.make_x(n, 3)
    y_ref, mag = ref.spmv(m, n, ti, tj, ta, x)
    for fmt in range(6):
        h = mo.mo_convert(a, fmt)
        Y = gpu_spmm(h, x.reshape(n, 1), m, np.float64)
        check(Y[:, 0], y_ref, mag, 1e-13, mo.FORMAT_NAMES[fmt])
        h.free()


def test_spmm_arguments():
    m, n, rp, ci, v = synth.config(1)
    a = upload(m, n, rp, ci, v)
    h = mo.mo_convert(a, mo.MO_CSR)
    x = torch.zeros((n, 65), dtype=torch.float64, device="cuda")
    y = torch.zeros((m, 65), dtype=torch.float64, device="cuda")
    with pytest.raises(mo.MoError) as e:
        mo.mo_spmm(h, x, y)
    assert e.value.status == mo.MO_E_PARAM
    with pytest.raises(mo.MoError) as e:
        mo.mo_tune_spmm(a, 0)
    assert e.value.status == mo.MO_E_PARAM


def test_tune_spmm():
    m, n, rp, ci, v = synth.config(2, 0.19)
    a = upload(m, n, rp, ci, v)
    best, ms, cv = mo.mo_tune_spmm(a, 4, warmups=2, reps=10)
    assert best == mo.mo_pick(ms) and not any(math.isnan(t) for t in ms)      # every format is feasible on the stencil
    assert all(t > 0 for t in ms) and all(t > 0 for t in cv)
    _, ms3, _ = mo.mo_tune_spmm(upload(*synth.config(3, 1 / 64)), 4, warmups=1, reps=3)
    assert math.isnan(ms3[mo.MO_DIA]) and math.isnan(ms3[mo.MO_ELL])
