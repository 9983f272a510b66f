"""Pins for the oracle's format -> triplets -> CSR direction (CPU only)."""
import numpy as np
import pytest

from oracle import ref
from paper_2303_05098_amd import synth
from tests import dense_pins
from tests.test_oracle_convert import CASES, shuffled, trip_set


def oracle_arrays(fmt, m, n, ti, tj, ta):
    if fmt == ref.FMT_COO:
        r, c, v = ref.to_coo(ti, tj, ta)
        return dict(coo_row=r, coo_col=c, coo_val=v)
    if fmt == ref.FMT_CSR:
        rp, c, v = ref.to_csr(m, ti, tj, ta)
        return dict(csr_row_ptr=rp, csr_col=c, csr_val=v)
    if fmt == ref.FMT_DIA:
        off, val = ref.to_dia(m, n, ti, tj, ta)
        return dict(dia_off=off, dia_val=val)
    if fmt == ref.FMT_ELL:
        k, col, val = ref.to_ell(m, ti, tj, ta)
        return dict(ell_col=col, ell_val=val)
    if fmt == ref.FMT_HYB:
        return ref.to_hyb(m, ti, tj, ta)
    return ref.to_hdc(m, n, ti, tj, ta)


@pytest.mark.parametrize("seed,m,n,dens,efrac", CASES)
def test_every_format_round_trips(seed, m, n, dens, efrac):
    m, n, rp, ci, v = synth.random_csr(m, n, dens, seed, efrac)
    ti, tj, ta = shuffled(seed, *ref.csr_to_triplets(rp, ci, v))
    want = trip_set(*ref.csr_to_triplets(rp, ci, v))
    for fmt in range(6):
        got = ref.format_to_triplets(fmt, m, n, oracle_arrays(fmt, m, n, ti, tj, ta))
        assert trip_set(*got) == want, fmt
        rp2, c2, v2 = ref.to_csr(m, *got)
        assert np.array_equal(rp2, rp) and np.array_equal(c2, ci) and np.array_equal(v2, v)


def test_to_csr_against_dense_definition():
    m, n, rp, ci, v = synth.random_csr(13, 9, 0.4, 3, 0.3)
    a, mask = dense_pins.dense_from_csr(m, n, rp, ci, v)
    ti, tj, ta = shuffled(3, *ref.csr_to_triplets(rp, ci, v))
    rp2, c2, v2 = ref.to_csr(m, ti, tj, ta)
    cols, vals, ptr = [], [], [0]
    for i in range(m):
        for j in range(n):
            if mask[i, j]:
                cols.append(j)
                vals.append(a[i, j])
        ptr.append(len(cols))
    assert list(rp2) == ptr and list(c2) == cols and list(v2) == vals


def test_dia_drops_zeros_and_out_of_matrix_positions_ell_keeps_stored_zeros():
    # 3 x 4, diagonals -1 and +2; one stored zero on diagonal +2
    off = np.array([-1, 2], np.int32)
    val = np.array([[9.0, 1.0, 2.0],        # row 0 has no column -1: the 9 sits outside the matrix
                    [3.0, 0.0, 7.0]])       # (0,2)=3, (1,3)=0 (not an entry), row 2 has no column 4
    ti, tj, ta = ref.from_dia(3, 4, off, val)
    assert trip_set(ti, tj, ta) == [(0, 2, 3.0), (1, 0, 1.0), (2, 1, 2.0)]
    col = np.array([[0, 2, -1], [3, -1, -1]], np.int32)
    ev = np.array([[5.0, 0.0, 0.0], [6.0, 0.0, 0.0]])
    ti, tj, ta = ref.from_ell(3, col, ev)
    assert trip_set(ti, tj, ta) == [(0, 0, 5.0), (0, 3, 6.0), (1, 2, 0.0)]


def test_features_from_any_format_equal_features_from_csr():
    m, n, rp, ci, v = synth.config(4, 1 / 512)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    want, wints = ref.features(m, n, ti, tj)
    for fmt in (0, 1, 3, 4, 5):
        got = ref.format_to_triplets(fmt, m, n, oracle_arrays(fmt, m, n, ti, tj, ta))
        f, ints = ref.features(m, n, got[0], got[1])
        assert f.tobytes() == want.tobytes() and ints == wints
