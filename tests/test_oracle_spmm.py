"""Pins for the oracle's multi-vector product Y = A X (CPU only): dense matrix products on tiny rectangular cases,
the identity that column v of Y is the (separately pinned) SpMV with column v of X, unit matrices, scipy."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import ref
from paper_2303_05098_amd import synth
from tests import dense_pins


def make_X(n, k, seed):
    return synth.uniform_pm1(seed, 40, np.arange(n * k)).reshape(n, k)


@pytest.mark.parametrize("seed,m,n,k,dens", [(1, 7, 5, 3, 0.4), (2, 16, 16, 1, 0.2), (3, 33, 64, 8, 0.1), (4, 64, 9, 5, 0.5), (5, 1, 40, 2, 0.5), (6, 40, 1, 4, 0.5)])
def test_dense_product(seed, m, n, k, dens):
    m, n, rp, ci, v = synth.random_csr(m, n, dens, seed, empty_row_frac=0.2)
    a, _ = dense_pins.dense_from_csr(m, n, rp, ci, v)
    X = make_X(n, k, seed)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    Y, mag = ref.spmm(m, n, ti, tj, ta, X)
    assert Y.shape == (m, k) and mag.shape == (m, k)
    assert np.allclose(Y, a @ X, rtol=0, atol=1e-14 * max(1, n))          # a transposed X (k x n read as n x k) fails here
    assert np.allclose(mag, np.abs(a) @ np.abs(X), rtol=1e-14, atol=0)


def test_columns_are_spmv():
    m, n, rp, ci, v = synth.config(4, 1 / 1024)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    X = make_X(n, 6, 3)
    Y, mag = ref.spmm(m, n, ti, tj, ta, X)
    for c in range(6):
        y, g = ref.spmv(m, n, ti, tj, ta, X[:, c])
        assert np.array_equal(Y[:, c], y) and np.array_equal(mag[:, c], g)     # same sums in the same order


def test_identity_and_scipy():
    n, k = 50, 7
    X = make_X(n, k, 9)
    eye = np.arange(n, dtype=np.int32)
    Y, _ = ref.spmm(n, n, eye, eye, np.ones(n), X)
    assert np.array_equal(Y, X)
    m, n, rp, ci, v = synth.random_csr(80, 60, 0.1, 21)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    X = make_X(n, 4, 10)
    Y, _ = ref.spmm(m, n, ti, tj, ta, X)
    assert np.allclose(Y, sp.csr_matrix((v, ci, rp), shape=(m, n)) @ X, rtol=0, atol=1e-13)
    with pytest.raises(ValueError):
        ref.spmm(3, 3, [0, 5], [0, 0], [1.0, 1.0], np.zeros((3, 2)))
