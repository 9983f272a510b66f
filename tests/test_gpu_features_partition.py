"""GPU parity of the feature call on matrices that take the partition path of the diagonal histogram (at least 2^21
entries on diagonals that adjacent rows do not share): the ten features bit for bit against the oracle (Table I), the
HDC conversion, which reads the per-diagonal counts, array by array, and arrays that violate the CSR precondition, which
must come back as MO_E_CSR_INVALID and leave the next call exact."""
import numpy as np
import pytest

from oracle import ref
from paper_2303_05098_amd import mo, synth
from tests.gpu_util import upload
from tests.test_gpu_parity import check_arrays

pytestmark = pytest.mark.gpu


def scattered(kind):
    if kind == "uniform":                 # 12 distinct uniform columns in every row
        return synth.uniform_rows(180000, 12, 91)
    if kind == "pow2":                    # 2^17 rows of 16: the bucket-by-block count table is a whole number of 256-byte lines
        return synth.uniform_rows(131072, 16, 97)
    if kind == "lognormal":               # rows of very different lengths, some empty, some beyond the lane-per-row limit
        return synth.lognormal_rows(140000, 92, mean=16.0, sigma=1.2)
    if kind == "wide":                    # more columns than rows
        m, n = 150000, 400000
        lens = np.full(m, 15, dtype=np.int64)
        rp, ci = synth._distinct_sorted_columns(lens, n, 93, 20)
        return m, n, rp, ci, synth.uniform_pm1(93, 12, np.arange(ci.shape[0], dtype=np.uint64))
    if kind == "tall":                    # more rows than columns, a stretch of empty rows in the middle
        m, n = 400000, 90000
        lens = np.full(m, 6, dtype=np.int64)
        lens[150000:158000] = 0
        rp, ci = synth._distinct_sorted_columns(lens, n, 94, 20)
        return m, n, rp, ci, synth.uniform_pm1(94, 12, np.arange(ci.shape[0], dtype=np.uint64))
    if kind == "with_diagonal":           # scattered columns plus the full main diagonal: one true diagonal
        m, n, rp, ci, v = synth.uniform_rows(170000, 12, 95)
        rows = np.repeat(np.arange(m, dtype=np.int64), np.diff(rp))
        keys = np.unique(np.concatenate([rows * n + ci.astype(np.int64), np.arange(m, dtype=np.int64) * (n + 1)]))
        r2, c2 = keys // n, keys % n
        rp2 = np.zeros(m + 1, np.int64)
        np.cumsum(np.bincount(r2, minlength=m), out=rp2[1:])
        return m, n, rp2.astype(np.int32), c2.astype(np.int32), synth.uniform_pm1(95, 13, np.arange(c2.shape[0], dtype=np.uint64))
    raise ValueError(kind)


@pytest.mark.parametrize("kind", ["uniform", "pow2", "lognormal", "wide", "tall", "with_diagonal"])
def test_features_bit_exact(kind):
    m, n, rp, ci, v = scattered(kind)
    assert ci.shape[0] >= 1 << 21
    a = upload(m, n, rp, ci, v)
    ti, tj, _ = ref.csr_to_triplets(rp, ci, v)
    for td in ((1, 2), (1, 100000), (1, 2)):      # the second call and the third reuse the scratch the first one left
        f, ints = mo.mo_features(a, dict(td_num=td[0], td_den=td[1]))
        fo, io = ref.features(m, n, ti, tj, td)
        assert f.tobytes() == fo.tobytes(), (f, fo)
        assert ints == io


def test_hdc_from_partitioned_counts():
    m, n, rp, ci, v = scattered("with_diagonal")
    a = upload(m, n, rp, ci, v)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    f, _ = mo.mo_features(a)
    assert f[9] == 1.0                             # the main diagonal is the one true diagonal
    h = mo.mo_convert(a, mo.MO_HDC)
    e = h.export()
    assert e["nd"] == 1
    check_arrays("with_diagonal", e, m, n, ti, tj, ta, None)
    h.free()
    with pytest.raises(mo.MoError) as err:         # 2 M diagonals of one or two entries: far beyond the padding limit
        mo.mo_convert(a, mo.MO_DIA)
    assert err.value.status == mo.MO_E_FILL


@pytest.mark.parametrize("kind", ["col_high", "col_negative", "col_unsorted", "rp_decreasing", "rp_beyond", "rp0", "rp_garbage"])
def test_invalid_arrays_are_rejected(kind):
    m, n, rp, ci, v = scattered("uniform")
    rp, ci = rp.copy(), ci.copy()
    mid = m // 2
    if kind == "col_high":
        ci[rp[mid] + 11] = n + 7
    elif kind == "col_negative":
        ci[rp[mid]] = -3
    elif kind == "col_unsorted":
        ci[rp[mid] + 4], ci[rp[mid] + 5] = ci[rp[mid] + 5], ci[rp[mid] + 4]
    elif kind == "rp_decreasing":
        rp[mid] = rp[mid - 1] - 5
    elif kind == "rp_beyond":
        rp[mid] = rp[-1] + 1000
    elif kind == "rp0":
        rp[0] = 3
    elif kind == "rp_garbage":                     # every row pointer but the last replaced by a seeded draw: no order at all
        draw = synth.bits64(96, 0, np.arange(m, dtype=np.uint64))
        rp[:m] = (draw % np.uint64(3 * int(rp[-1])) - np.uint64(int(rp[-1]))).astype(np.int64).astype(np.int32)
    a = upload(m, n, rp, ci, v)
    for _ in range(2):
        with pytest.raises(mo.MoError) as e:
            mo.mo_features(a)
        assert e.value.status == mo.MO_E_CSR_INVALID
    with pytest.raises(mo.MoError) as e:
        mo.mo_convert(a, mo.MO_HDC)
    assert e.value.status == mo.MO_E_CSR_INVALID
    # and the kept scratch serves the next valid matrix exactly
    m2, n2, rp2, ci2, v2 = scattered("wide")
    f, ints = mo.mo_features(upload(m2, n2, rp2, ci2, v2))
    ti, tj, _ = ref.csr_to_triplets(rp2, ci2, v2)
    fo, io = ref.features(m2, n2, ti, tj)
    assert f.tobytes() == fo.tobytes() and ints == io
