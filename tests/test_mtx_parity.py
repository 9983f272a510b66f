"""The library's Matrix Market reader (mo_mtx_read, host code) against the oracle: same CSR arrays bit for bit on
files of every supported kind, and a refusal wherever the oracle refuses."""
import numpy as np
import pytest
import scipy.io
import scipy.sparse as sp

from oracle import mtx
from paper_2303_05098_amd import mo, synth
from tests.test_oracle_mtx import test_refusals as _refusal_cases

REFUSALS = [p.values[0] if hasattr(p, "values") else p for p in _refusal_cases.pytestmark[0].args[1]]


def same_as_oracle(path):
    m, n, rp, ci, v = mo.mo_mtx_read(path)
    om, on, orp, oci, ov = mtx.read_csr(path)
    assert (m, n) == (om, on)
    assert rp.tolist() == orp and ci.tolist() == oci
    assert v.tobytes() == np.asarray(ov, dtype=np.float64).tobytes()
    return m, n, rp, ci, v


@pytest.mark.parametrize("symmetry", ["general", "symmetric", "skew-symmetric"])
@pytest.mark.parametrize("field", ["real", "integer", "pattern"])
def test_scipy_written_files(tmp_path, symmetry, field):
    mm, n, rp, ci, v = synth.random_csr(300, 300, 0.03, 9, 0.1)
    a = sp.csr_matrix((v, ci, rp), shape=(mm, n))
    if field != "real":
        a.data = np.round(a.data * 10)
        a.data[a.data == 0] = 3
    if symmetry == "symmetric":
        a = a + a.T
    if symmetry == "skew-symmetric":
        a = sp.triu(a, 1) - sp.triu(a, 1).T
    p = str(tmp_path / "s.mtx")
    scipy.io.mmwrite(p, a.tocoo(), field=field, symmetry=symmetry, precision=17)
    same_as_oracle(p)


def test_round_trip_of_a_synthetic_matrix(tmp_path):
    m, n, rp, ci, v = synth.config(4, 1 / 512)
    p = str(tmp_path / "c4.mtx")
    scipy.io.mmwrite(p, sp.csr_matrix((v, ci, rp), shape=(m, n)).tocoo(), precision=17)
    m2, n2, rp2, ci2, v2 = same_as_oracle(p)
    assert (m2, n2) == (m, n) and np.array_equal(rp2, rp) and np.array_equal(ci2, ci) and v2.tobytes() == v.tobytes()


def test_hand_written_files(tmp_path):
    texts = [
        "%%MatrixMarket MATRIX Coordinate Real General\n% a comment\n\n%another\n  3 4   6\n1 1 1.5\n3 4 -2e0\n2 2 0\n1 1 2.5\n3 1 7\n\n1 3 1e-3\n",
        "%%MatrixMarket matrix coordinate integer symmetric\r\n2 2 2\r\n2 1 5\r\n2 2 9\r\n",
        "%%MatrixMarket matrix coordinate real skew-symmetric\n3 3 2\n2 1 5\n3 1 -0.25",
        "%%MatrixMarket matrix coordinate pattern general\n2 3 2\n1 3\n2 1\n",
        "%%MatrixMarket matrix coordinate real general\n5 5 0\n",
        "%%MatrixMarket matrix coordinate real general\n2 2 4\n1 1 0.1\n1 1 0.2\n1 1 0.3\n1 1 1e100\n",        # summation order matters
        "%%MatrixMarket matrix coordinate real symmetric\n2 2 3\n2 1 0.1\n1 2 0.2\n2 1 0.3\n",                   # both triangles present
        "%%MatrixMarket matrix coordinate real general\n1 1 1\n\t1\t1\t+.5e+1  \n\n\n",
    ]
    for k, text in enumerate(texts):
        p = tmp_path / f"h{k}.mtx"
        p.write_bytes(text.encode())
        same_as_oracle(str(p))


@pytest.mark.parametrize("text", REFUSALS)
def test_refusals(tmp_path, text):
    p = tmp_path / "bad.mtx"
    p.write_bytes(text.encode())
    with pytest.raises((mtx.MtxError, ValueError)):
        mtx.read_triplets(str(p))
    with pytest.raises(mo.MoError) as e:
        mo.mo_mtx_read(str(p))
    assert e.value.status == mo.MO_E_IO


def test_missing_file(tmp_path):
    with pytest.raises(mo.MoError) as e:
        mo.mo_mtx_read(str(tmp_path / "nope.mtx"))
    assert e.value.status == mo.MO_E_IO
