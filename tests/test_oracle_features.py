"""Pins for the oracle's ten features (Table I) — CPU only."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref
from paper_2303_05098_amd import synth
from tests import dense_pins
from tests.test_oracle_spmv import gold


def test_c1_closed_form():
    g = gold()
    m, n, rp, ci, v = synth.config(1)
    ti, tj, _ = ref.csr_to_triplets(rp, ci, v)
    f, ints = ref.features(m, n, ti, tj)
    assert f[0] == g["m"] and f[1] == g["n"] and f[2] == g["nnz"]
    assert f[3] == g["avg"]
    assert f[4] == 20224 / (4096 * 4096)
    assert f[5] == g["max_row"] and f[6] == g["min_row"]
    assert ints["sum_sq_row"] == g["sum_sq_row"]
    assert f[7] == math.sqrt(g["variance"])
    assert abs(f[7] - g["std"]) < 1e-13
    assert f[8] == g["n_diag"] and f[9] == g["n_true_diag"]


def stencil27_closed_form(g):
    """Row-length classes and diagonal counts of the 27-point stencil on g^3."""
    inner, face = g - 2, 2
    # per axis: (g-2) coordinates see 3 neighbours, 2 see 2
    counts = {}
    for ax, nx in ((3, inner), (2, face)):
        for ay, ny in ((3, inner), (2, face)):
            for az, nz in ((3, inner), (2, face)):
                counts[ax * ay * az] = counts.get(ax * ay * az, 0) + nx * ny * nz
    nnz = (3 * g - 2) ** 3
    sumsq = sum(k * k * c for k, c in counts.items())
    diag = {}
    for dz in (-1, 0, 1):
        for dy in (-1, 0, 1):
            for dx in (-1, 0, 1):
                diag[(dz * g + dy) * g + dx] = (g - abs(dx)) * (g - abs(dy)) * (g - abs(dz))
    return counts, nnz, sumsq, diag


@pytest.mark.parametrize("g", [4, 7, 16])
def test_stencil27_closed_form(g):
    m, n, rp, ci, v = synth.stencil27(g, 3)
    counts, nnz, sumsq, diag = stencil27_closed_form(g)
    assert rp[-1] == nnz
    ti, tj, _ = ref.csr_to_triplets(rp, ci, v)
    f, ints = ref.features(m, n, ti, tj)
    assert ints["nnz"] == nnz and ints["sum_sq_row"] == sumsq
    assert f[5] == 27 and f[6] == 8
    assert f[3] == nnz / m
    var = Fraction(m * sumsq - nnz * nnz, m * m)
    assert abs(f[7] - math.sqrt(var)) <= 2e-16 * math.sqrt(var)
    assert f[8] == len(diag)
    assert f[9] == sum(1 for c in diag.values() if 2 * c >= m)


def test_stencil27_full_size_numbers():
    # the 128^3 closed forms quoted for the large stencil configuration
    counts, nnz, sumsq, diag = stencil27_closed_form(128)
    assert nnz == 55742968 and sumsq == 1489355288
    assert counts == {27: 2000376, 18: 95256, 12: 1512, 8: 8}
    assert min(diag.values()) == 2048383 and max(diag.values()) == 2097152 and len(diag) == 27


def test_band_only_diagonals():
    m = 8192
    mm, n, rp, ci, v = synth.banded_scatter(m, synth.C4_OFFSETS, 0, 100, 1)
    ti, tj, _ = ref.csr_to_triplets(rp, ci, v)
    f, ints = ref.features(m, n, ti, tj)
    assert ints["nnz"] == 9 * m - 2 * (1 + 2 + 2048 + 4096)
    assert f[8] == 9
    # |d| = 4096 diagonals hold m - 4096 = 4096 entries = exactly half of min(M,N): still true (>=)
    assert f[9] == 9
    f2, _ = ref.features(m, n, ti, tj, td=(4097, 8192))
    assert f2[9] == 7


@pytest.mark.parametrize("seed,m,n,dens,efrac", [(1, 9, 9, 0.3, 0.0), (2, 12, 7, 0.3, 0.3), (3, 5, 17, 0.5, 0.2),
                                                 (4, 30, 30, 0.05, 0.0), (5, 1, 6, 0.7, 0.0), (6, 6, 1, 0.7, 0.0)])
def test_bruteforce_dense(seed, m, n, dens, efrac):
    m, n, rp, ci, v = synth.random_csr(m, n, dens, seed, efrac)
    a, mask = dense_pins.dense_from_csr(m, n, rp, ci, v)
    ti, tj, _ = ref.csr_to_triplets(rp, ci, v)
    for td in ((1, 2), (1, 4), (1, 1)):
        f, _ = ref.features(m, n, ti, tj, td)
        want = dense_pins.features(a, mask, td)
        for k in range(10):
            if k == 7:
                assert abs(f[k] - want[k]) <= 1e-14 * max(1.0, want[k])
            else:
                assert f[k] == want[k], (k, f[k], want[k])


def test_identity_and_single_dense_row_and_empty():
    n = 50
    ti = np.arange(n, dtype=np.int32)
    f, _ = ref.features(n, n, ti, ti)
    assert list(f) == [n, n, n, 1.0, 1.0 / n, 1, 1, 0.0, 1, 1]
    # one dense row in an otherwise empty 10 x 8 matrix
    ti = np.full(8, 3, np.int32)
    tj = np.arange(8, dtype=np.int32)
    f, ints = ref.features(10, 8, ti, tj)
    assert f[2] == 8 and f[5] == 8 and f[6] == 0 and f[8] == 8 and f[9] == 0
    assert abs(f[7] - math.sqrt((9 * 0.8 ** 2 + 7.2 ** 2) / 10)) < 1e-15
    # no entries at all
    f, _ = ref.features(4, 5, np.zeros(0, np.int32), np.zeros(0, np.int32))
    assert list(f) == [4, 5, 0, 0.0, 0.0, 0, 0, 0.0, 0, 0]


def test_stored_zero_counts_as_entry():
    f, _ = ref.features(2, 2, [0, 1], [0, 1])
    assert f[2] == 2 and f[8] == 1
