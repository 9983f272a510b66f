"""Pins for the oracle's SpMV (CPU only)."""
import os

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import ref
from paper_2303_05098_amd import synth
from tests import dense_pins

GOLD = os.path.join(os.path.dirname(__file__), "golden", "c1_laplace64.txt")


def gold():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        out[k] = float(v)
    return out


@pytest.mark.parametrize("seed,m,n,dens", [(1, 7, 5, 0.4), (2, 16, 16, 0.2), (3, 33, 64, 0.1), (4, 64, 9, 0.5), (5, 1, 40, 0.5), (6, 40, 1, 0.5)])
def test_dense_matvec(seed, m, n, dens):
    m, n, rp, ci, v = synth.random_csr(m, n, dens, seed, empty_row_frac=0.2)
    a, mask = dense_pins.dense_from_csr(m, n, rp, ci, v)
    x = synth.make_x(n, seed)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    y, mag = ref.spmv(m, n, ti, tj, ta, x)
    assert np.allclose(y, a @ x, rtol=0, atol=1e-14 * max(1, n))
    assert np.allclose(mag, np.abs(a) @ np.abs(x), rtol=1e-14, atol=0)
    # a transposed operand or swapped index would break rectangular cases above; also check order invariance
    perm = np.argsort(synth.uniform01(seed, 99, np.arange(ti.shape[0])))
    y2, _ = ref.spmv(m, n, ti[perm], tj[perm], ta[perm], x)
    assert np.allclose(y2, y, rtol=0, atol=1e-15 * max(1, n))


def test_unit_vectors_give_columns():
    m, n, rp, ci, v = synth.random_csr(12, 9, 0.4, 11)
    a, _ = dense_pins.dense_from_csr(m, n, rp, ci, v)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    for j in range(n):
        e = np.zeros(n)
        e[j] = 1.0
        y, _ = ref.spmv(m, n, ti, tj, ta, e)
        assert np.array_equal(y, a[:, j])


def test_laplace_rowsums_closed_form():
    g = gold()
    m, n, rp, ci, v = synth.config(1)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    y, mag = ref.spmv(m, n, ti, tj, ta, np.ones(n))
    r = np.arange(m)
    ix, iy = r % 64, r // 64
    nb = (ix == 0).astype(int) + (ix == 63) + (iy == 0) + (iy == 63)
    assert np.array_equal(y[nb == 0], np.full((nb == 0).sum(), g["rowsum_interior"]))
    assert np.array_equal(y[nb == 1], np.full((nb == 1).sum(), g["rowsum_edge"]))
    assert np.array_equal(y[nb == 2], np.full((nb == 2).sum(), g["rowsum_corner"]))
    assert (nb == 0).sum() == 3844 and (nb == 1).sum() == 248 and (nb == 2).sum() == 4
    assert np.array_equal(mag, 8.0 - nb)


@pytest.mark.parametrize("c,scale", [(2, 0.1), (3, 1 / 256), (4, 1 / 256)])
def test_against_scipy(c, scale):
    m, n, rp, ci, v = synth.config(c, scale)
    x = synth.make_x(n, synth.BASE_SEED + c)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    y, mag = ref.spmv(m, n, ti, tj, ta, x)
    ys = sp.csr_matrix((v, ci, rp), shape=(m, n)) @ x
    err, zeros_ok = ref.spmv_error(ys, y, mag)
    assert err <= 1e-13 and zeros_ok


def test_linearity():
    m, n, rp, ci, v = synth.config(3, 1 / 512)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    x, z = synth.make_x(n, 1), synth.make_x(n, 2)
    yx, magx = ref.spmv(m, n, ti, tj, ta, x)
    yz, magz = ref.spmv(m, n, ti, tj, ta, z)
    yc, _ = ref.spmv(m, n, ti, tj, ta, 2.0 * x - 3.0 * z)
    bound = 1e-14 * (2 * magx + 3 * magz) + 1e-300
    assert np.all(np.abs(yc - (2.0 * yx - 3.0 * yz)) <= bound)


def test_extended_accumulation_beats_plain_double():
    # one row: 1 + many tiny terms that plain fp64 accumulation would drop entirely
    k = 4096
    ti = np.zeros(k + 1, np.int32)
    tj = np.arange(k + 1, dtype=np.int32)
    ta = np.concatenate([[1.0], np.full(k, 2.0 ** -54)])
    y, _ = ref.spmv(1, k + 1, ti, tj, ta, np.ones(k + 1))
    assert y[0] == 1.0 + k * 2.0 ** -54


def test_multithreaded_variant_matches():
    m, n, rp, ci, v = synth.config(3, 1 / 128)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    x = synth.make_x(n, 5)
    y, _ = ref.spmv(m, n, ti, tj, ta, x)
    for nt in (1, 3, 8):
        assert np.array_equal(ref.spmv_rowsorted_mt(m, ti, tj, ta, x, nt), y)


def test_rejects_out_of_range():
    with pytest.raises(ValueError):
        ref.spmv(2, 2, [0, 2], [0, 1], [1.0, 1.0], np.ones(2))
    with pytest.raises(ValueError):
        ref.spmv(2, 2, [0, 1], [0, 2], [1.0, 1.0], np.ones(2))
