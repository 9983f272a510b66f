"""Pins for the oracle's format conversions (Section II-B) — CPU only."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import ref
from paper_2303_05098_amd import synth
from tests import dense_pins
from tests.test_oracle_spmv import gold

CASES = [(1, 9, 9, 0.3, 0.0), (2, 12, 7, 0.3, 0.3), (3, 5, 17, 0.5, 0.2), (4, 30, 30, 0.05, 0.0),
         (5, 1, 6, 0.7, 0.0), (6, 6, 1, 0.7, 0.0), (7, 24, 24, 0.6, 0.1)]


def trip_set(ti, tj, ta):
    return sorted(zip(map(int, ti), map(int, tj), map(float, ta)))


def shuffled(seed, ti, tj, ta):
    perm = np.argsort(synth.uniform01(seed, 98, np.arange(ti.shape[0])))
    return ti[perm], tj[perm], ta[perm]


@pytest.mark.parametrize("seed,m,n,dens,efrac", CASES)
def test_coo_sorted(seed, m, n, dens, efrac):
    m, n, rp, ci, v = synth.random_csr(m, n, dens, seed, efrac)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    r, c, a = ref.to_coo(*shuffled(seed, ti, tj, ta))
    assert np.array_equal(r, ti) and np.array_equal(c, tj) and np.array_equal(a, ta)


@pytest.mark.parametrize("seed,m,n,dens,efrac", CASES)
def test_dia_bruteforce(seed, m, n, dens, efrac):
    m, n, rp, ci, v = synth.random_csr(m, n, dens, seed, efrac)
    a, mask = dense_pins.dense_from_csr(m, n, rp, ci, v)
    ti, tj, ta = shuffled(seed, *ref.csr_to_triplets(rp, ci, v))
    off, val = ref.to_dia(m, n, ti, tj, ta)
    woff, wval = dense_pins.dia(a, mask)
    assert np.array_equal(off, woff) and np.array_equal(val, wval)
    f, _ = ref.features(m, n, ti, tj)
    assert off.shape[0] == f[8]
    # library cross-check of the offset set
    so = np.sort(sp.csr_matrix((np.ones_like(v), ci, rp), shape=(m, n)).todia().offsets)
    assert np.array_equal(so, off)


@pytest.mark.parametrize("seed,m,n,dens,efrac", CASES)
def test_ell_bruteforce(seed, m, n, dens, efrac):
    m, n, rp, ci, v = synth.random_csr(m, n, dens, seed, efrac)
    a, mask = dense_pins.dense_from_csr(m, n, rp, ci, v)
    ti, tj, ta = shuffled(seed, *ref.csr_to_triplets(rp, ci, v))
    k, col, val = ref.to_ell(m, ti, tj, ta)
    wk, wcol, wval, rest = dense_pins.ell(a, mask)
    assert k == wk and not rest
    assert np.array_equal(col, wcol) and np.array_equal(val, wval)
    assert (col >= 0).sum() == rp[-1]
    f, _ = ref.features(m, n, ti, tj)
    assert k == f[5]


@pytest.mark.parametrize("seed,m,n,dens,efrac", CASES)
@pytest.mark.parametrize("hyb", [(1, 3), (1, 2), (1, 1), (0, 1), (2, 1)])
def test_hyb_bruteforce(seed, m, n, dens, efrac, hyb):
    m, n, rp, ci, v = synth.random_csr(m, n, dens, seed, efrac)
    a, mask = dense_pins.dense_from_csr(m, n, rp, ci, v)
    ti, tj, ta = shuffled(seed, *ref.csr_to_triplets(rp, ci, v))
    h = ref.to_hyb(m, ti, tj, ta, hyb)
    wk = dense_pins.hyb_k(mask, hyb)
    assert h["k"] == wk
    _, wcol, wval, rest = dense_pins.ell(a, mask, wk)
    assert np.array_equal(h["ell_col"], wcol) and np.array_equal(h["ell_val"], wval)
    assert trip_set(h["coo_row"], h["coo_col"], h["coo_val"]) == [(i, j, float(x)) for i, j, x in rest]
    assert list(zip(h["coo_row"], h["coo_col"])) == sorted(zip(h["coo_row"], h["coo_col"]))
    assert (h["ell_col"] >= 0).sum() + h["coo_row"].shape[0] == rp[-1]


def test_hyb_k_hand_histograms():
    # lengths 5,5,5,1,1,1,1,1,0: 3 of 9 rows reach 5 -> K_H = 5 at 1/3; 8 of 9 reach 1 -> K_H = 1 at 1/2
    lens = [5, 5, 5, 1, 1, 1, 1, 1, 0]
    ti = np.repeat(np.arange(9, dtype=np.int32), lens)
    assert ref.hyb_k(9, ti, (1, 3)) == 5
    assert ref.hyb_k(9, ti, (1, 2)) == 1
    assert ref.hyb_k(9, ti, (1, 1)) == 0
    assert ref.hyb_k(9, ti, (8, 9)) == 1
    assert ref.hyb_k(9, ti, (0, 1)) == 5          # every k qualifies -> max length
    assert ref.hyb_k(9, ti, (10, 9)) == 0         # even k = 0 does not qualify -> 0
    ks = [ref.hyb_k(9, ti, (p, 9)) for p in range(0, 10)]
    assert ks == sorted(ks, reverse=True)         # raising the fraction never raises K_H


@pytest.mark.parametrize("seed,m,n,dens,efrac", CASES)
@pytest.mark.parametrize("td", [(1, 2), (1, 4), (1, 8), (1, 1)])
def test_hdc_bruteforce(seed, m, n, dens, efrac, td):
    m, n, rp, ci, v = synth.random_csr(m, n, dens, seed, efrac)
    a, mask = dense_pins.dense_from_csr(m, n, rp, ci, v)
    ti, tj, ta = shuffled(seed, *ref.csr_to_triplets(rp, ci, v))
    h = ref.to_hdc(m, n, ti, tj, ta, td)
    woff, wval, wrp, wcol, wv = dense_pins.hdc(a, mask, td)
    assert np.array_equal(h["dia_off"], woff) and np.array_equal(h["dia_val"], wval)
    assert np.array_equal(h["csr_row_ptr"], wrp)
    assert np.array_equal(h["csr_col"], wcol) and np.array_equal(h["csr_val"], wv)
    f, _ = ref.features(m, n, ti, tj, td)
    assert h["dia_off"].shape[0] == f[9]


def test_c1_conversion_closed_forms():
    g = gold()
    m, n, rp, ci, v = synth.config(1)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    off, val = ref.to_dia(m, n, ti, tj, ta)
    assert list(off) == [-64, -1, 0, 1, 64]
    assert val.size - np.count_nonzero(val) == g["dia_padding"]
    assert np.all(val[2] == 4.0)
    k, col, eval_ = ref.to_ell(m, ti, tj, ta)
    assert k == g["ell_k"] and (col < 0).sum() == g["ell_padding"]
    h = ref.to_hyb(m, ti, tj, ta)
    assert h["k"] == g["hyb_k"] and h["coo_row"].shape[0] == g["hyb_coo_nnz"]
    d = ref.to_hdc(m, n, ti, tj, ta)
    assert d["csr_col"].shape[0] == g["hdc_csr_nnz"] and list(d["dia_off"]) == [-64, -1, 0, 1, 64]
    assert np.all(d["csr_row_ptr"] == 0)


@pytest.mark.parametrize("c,scale", [(2, 0.08), (3, 1 / 1024), (4, 1 / 512)])
def test_round_trips(c, scale):
    m, n, rp, ci, v = synth.config(c, scale)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    want = trip_set(ti, tj, ta)
    # DIA
    keys = np.sort(ti.astype(np.int64) * n + tj)

    def dia_triplets(off, val):
        i = np.broadcast_to(np.arange(m, dtype=np.int64)[None, :], val.shape)
        j = i + off.astype(np.int64)[:, None]
        ok = (j >= 0) & (j < n)
        ok &= np.isin(i * n + j, keys)
        return trip_set(i[ok], j[ok], val[ok])

    off, val = ref.to_dia(m, n, ti, tj, ta)
    assert dia_triplets(off, val) == want
    assert np.count_nonzero(val) <= len(want)
    # ELL
    k, col, ev = ref.to_ell(m, ti, tj, ta)
    ks, is_ = np.nonzero(col >= 0)
    assert trip_set(is_, col[ks, is_], ev[ks, is_]) == want
    # HYB
    h = ref.to_hyb(m, ti, tj, ta)
    ks, is_ = np.nonzero(h["ell_col"] >= 0)
    got = trip_set(is_, h["ell_col"][ks, is_], h["ell_val"][ks, is_]) + trip_set(h["coo_row"], h["coo_col"], h["coo_val"])
    assert sorted(got) == want
    # HDC: parts disjoint and complete
    d = ref.to_hdc(m, n, ti, tj, ta)
    ri = np.repeat(np.arange(m), np.diff(d["csr_row_ptr"]))
    rest = trip_set(ri, d["csr_col"], d["csr_val"])
    dia_part = dia_triplets(d["dia_off"], d["dia_val"])
    assert not (set((i, j) for i, j, _ in rest) & set((i, j) for i, j, _ in dia_part))
    assert sorted(rest + dia_part) == want


def test_empty_matrix_conversions():
    z = np.zeros(0, np.int32)
    zf = np.zeros(0)
    off, val = ref.to_dia(3, 4, z, z, zf)
    assert off.shape == (0,) and val.shape == (0, 3)
    k, col, ev = ref.to_ell(3, z, z, zf)
    assert k == 0 and col.shape == (0, 3)
    h = ref.to_hyb(3, z, z, zf)
    assert h["k"] == 0 and h["coo_row"].shape[0] == 0
    d = ref.to_hdc(3, 4, z, z, zf)
    assert d["dia_off"].shape[0] == 0 and list(d["csr_row_ptr"]) == [0, 0, 0, 0]


def test_feasibility_rule():
    assert ref.feasible(16 * 10, 10)
    assert not ref.feasible(16 * 10 + 1, 10)
    assert ref.feasible(0, 0)
    assert not ref.feasible(100, 10, max_fill=16, max_slots=99)
