"""Pins of the Matrix Market oracle: files written by scipy.io.mmwrite and read back by scipy.io.mmread (an
independent implementation of the format), hand-written files with every feature of the format, and refusals."""
import numpy as np
import pytest
import scipy.io
import scipy.sparse as sp

from oracle import mtx
from paper_2303_05098_amd import synth


def write(tmp_path, text, name="a.mtx"):
    p = tmp_path / name
    p.write_text(text)
    return str(p)


def dense_of(m, n, rows, cols, vals):
    d = np.zeros((m, n))
    for i, j, v in zip(rows, cols, vals):
        d[i, j] = v
    return d


@pytest.mark.parametrize("symmetry", ["general", "symmetric", "skew-symmetric"])
@pytest.mark.parametrize("field", ["real", "integer", "pattern"])
def test_against_scipy(tmp_path, symmetry, field):
    mm, n, rp, ci, v = synth.random_csr(40, 40, 0.15, 5, 0.1)
    a = sp.csr_matrix((v, ci, rp), shape=(mm, n))
    if field != "real":
        a.data = np.round(a.data * 10)
        a.data[a.data == 0] = 3
    if symmetry == "symmetric":
        a = a + a.T
    if symmetry == "skew-symmetric":
        a = sp.triu(a, 1) - sp.triu(a, 1).T
    p = str(tmp_path / "s.mtx")
    scipy.io.mmwrite(p, a.tocoo(), field=field, symmetry=symmetry)
    want = scipy.io.mmread(p).toarray()
    got = dense_of(*mtx.read_triplets(p))
    assert np.array_equal(got, want)
    m2, n2, rp2, ci2, v2 = mtx.read_csr(p)
    b = sp.csr_matrix((v2, ci2, rp2), shape=(m2, n2))
    assert np.array_equal(b.toarray(), want) and b.has_sorted_indices


def test_hand_written_file(tmp_path):
    text = """%%MatrixMarket MATRIX Coordinate Real General
% a comment

%another
  3 4   6
1 1 1.5
3 4 -2e0
2 2 0
1 1 2.5
3 1 7

1 3 1e-3
"""
    m, n, r, c, v = mtx.read_triplets(write(tmp_path, text))
    # duplicates of (1,1) are summed, the explicit zero stays, order is (row, col)
    assert (m, n) == (3, 4)
    assert list(zip(r, c, v)) == [(0, 0, 4.0), (0, 2, 1e-3), (1, 1, 0.0), (2, 0, 7.0), (2, 3, -2.0)]
    assert mtx.read_csr(write(tmp_path, text))[2] == [0, 2, 3, 5]
    sym = "%%MatrixMarket matrix coordinate integer symmetric\n2 2 2\n2 1 5\n2 2 9\n"
    assert list(zip(*mtx.read_triplets(write(tmp_path, sym))[2:])) == [(0, 1, 5.0), (1, 0, 5.0), (1, 1, 9.0)]
    skew = "%%MatrixMarket matrix coordinate real skew-symmetric\n2 2 1\n2 1 5\n"
    assert list(zip(*mtx.read_triplets(write(tmp_path, skew))[2:])) == [(0, 1, -5.0), (1, 0, 5.0)]
    pat = "%%MatrixMarket matrix coordinate pattern general\n2 3 2\n1 3\n2 1\n"
    assert list(zip(*mtx.read_triplets(write(tmp_path, pat))[2:])) == [(0, 2, 1.0), (1, 0, 1.0)]
    empty = "%%MatrixMarket matrix coordinate real general\n5 5 0\n"
    assert mtx.read_csr(write(tmp_path, empty)) == (5, 5, [0] * 6, [], [])


@pytest.mark.parametrize("text", [
    "",                                                                         # no banner
    "%MatrixMarket matrix coordinate real general\n1 1 0\n",                     # one % only
    "%%MatrixMarket matrix array real general\n1 1\n1.0\n",                      # dense format
    "%%MatrixMarket matrix coordinate complex general\n1 1 1\n1 1 1 0\n",        # complex
    "%%MatrixMarket matrix coordinate real hermitian\n1 1 0\n",                  # hermitian
    "%%MatrixMarket matrix coordinate real general\n2 2\n",                      # short size line
    "%%MatrixMarket matrix coordinate real general\n2 2 2\n1 1 1\n",             # fewer entries than announced
    "%%MatrixMarket matrix coordinate real general\n2 2 1\n1 1 1\n2 2 2\n",      # more entries than announced
    "%%MatrixMarket matrix coordinate real general\n2 2 1\n3 1 1\n",             # row out of range
    "%%MatrixMarket matrix coordinate real general\n2 2 1\n1 0 1\n",             # column 0 (indices are 1-based)
    "%%MatrixMarket matrix coordinate real general\n2 2 1\n1 1\n",               # missing value
    "%%MatrixMarket matrix coordinate pattern general\n2 2 1\n1 1 1\n",          # value in a pattern file
    "%%MatrixMarket matrix coordinate real symmetric\n2 3 0\n",                  # symmetric but not square
    "%%MatrixMarket matrix coordinate real skew-symmetric\n2 2 1\n1 1 4\n",      # diagonal entry in a skew file
    "%%MatrixMarket matrix coordinate real general\n0 2 0\n",                    # empty dimension
])
def test_refusals(tmp_path, text):
    with pytest.raises((mtx.MtxError, ValueError)):
        mtx.read_triplets(write(tmp_path, text))
