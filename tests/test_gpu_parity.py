"""GPU parity: HIP library vs CPU oracle through the C ABI, element by element, on seeded inputs that span
several tiles and a ragged tail; plus the edge cases of every call."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2303_05098_amd import mo, synth
from tests.gpu_util import TOL, gpu_spmv, oracle_inputs, try_convert, upload

pytestmark = pytest.mark.gpu


def very_long_rows():
    """Two rows of 12 000 and 9 000 entries (every other column, every third) among rows of two: longer than what the
    feature traversal walks where it meets them, so they go through its list of deferred rows."""
    m, n, rp, ci, v = synth.uniform_rows(30000, 2, 19)
    lens = np.diff(rp).astype(np.int64)
    lens[700], lens[20001] = 12000, 9000
    rp2 = np.zeros(m + 1, np.int64)
    np.cumsum(lens, out=rp2[1:])
    ci2 = np.concatenate([ci[:rp[700]], np.arange(12000, dtype=np.int32) * 2 + 1, ci[rp[701]:rp[20001]],
                          np.arange(9000, dtype=np.int32) * 3, ci[rp[20002]:]])
    return m, n, rp2.astype(np.int32), ci2.astype(np.int32), synth.uniform_pm1(19, 0, np.arange(ci2.shape[0]))


def small_cases():
    """(name, m, n, row_ptr, col_idx, val) — sizes the oracle finishes in seconds."""
    out = [("c1", *synth.config(1)),
           ("c2s", *synth.config(2, 0.19)),          # 24^3 = 13824 rows, 27-point
           ("c3s", *synth.config(3, 1 / 64)),        # 16384 rows lognormal, long rows cross tiles
           ("c4s", *synth.config(4, 1 / 64)),        # 65536 rows banded + scatter
           ("uni", *synth.uniform_rows(5000, 3, 77)),
           ("rect_wide", *synth.random_csr(300, 1000, 0.02, 5, 0.3)),
           ("rect_tall", *synth.random_csr(1000, 130, 0.05, 6, 0.1)),
           ("one_row", *synth.random_csr(1, 5000, 0.7, 7)),
           ("one_col", *synth.random_csr(700, 1, 0.5, 8)),
           ("dense", *synth.random_csr(70, 70, 1.1, 9)),
           ("tiny", *synth.random_csr(3, 3, 0.5, 10))]
    # empty matrix and a matrix whose only entries sit in the last row
    out.append(("empty", 5, 7, np.zeros(6, np.int32), np.zeros(0, np.int32), np.zeros(0)))
    out.append(("last_row", 4000, 4000, np.concatenate([np.zeros(4000, np.int32), [3]]).astype(np.int32),
                np.array([0, 17, 3999], np.int32), np.array([1.0, -2.0, 0.5])))
    # one very long row between short ones (crosses many COO/CSR tiles)
    m, n, rp, ci, v = synth.uniform_rows(3000, 2, 12)
    lens = np.diff(rp).astype(np.int64)
    lens[1500] = 3000
    rp2 = np.zeros(m + 1, np.int64)
    np.cumsum(lens, out=rp2[1:])
    ci2 = np.concatenate([ci[:rp[1500]], np.arange(3000, dtype=np.int32), ci[rp[1501]:]])
    v2 = synth.uniform_pm1(13, 0, np.arange(ci2.shape[0]))
    out.append(("long_row", m, n, rp2.astype(np.int32), ci2.astype(np.int32), v2))
    out.append(("very_long_rows", *very_long_rows()))
    # the same with the full main diagonal and the diagonal above it: HDC keeps two true diagonals, and the long rows,
    # which hold entries on both of them, go to the chip-wide fill kernels of the DIA part and of the CSR remainder
    m, n, rp, ci, v = very_long_rows()
    rows = np.repeat(np.arange(m, dtype=np.int64), np.diff(rp))
    d = np.arange(m, dtype=np.int64)
    keys = np.unique(np.concatenate([rows * n + ci.astype(np.int64), d * (n + 1), d[:-1] * (n + 1) + 1]))
    r2, c2 = keys // n, keys % n
    rp2 = np.zeros(m + 1, np.int64)
    np.cumsum(np.bincount(r2, minlength=m), out=rp2[1:])
    out.append(("arrow", m, n, rp2.astype(np.int32), c2.astype(np.int32), synth.uniform_pm1(20, 0, np.arange(c2.shape[0]))))
    # a tridiagonal matrix with a 256-row stretch of 29 diagonals: the mean row is short, so a wave takes 64 rows, and in
    # the stretch their entries exceed one LDS stage of the conversion kernels (rows past the staged window)
    m = n = 4096
    rows, cols = [], []
    for i in range(m):
        reach = 14 if 1024 <= i < 1280 else 1
        js = np.arange(max(0, i - reach), min(n, i + reach + 1))
        rows.append(np.full(js.size, i))
        cols.append(js)
    ti, tj = np.concatenate(rows), np.concatenate(cols)
    rp3 = np.zeros(m + 1, np.int64)
    np.cumsum(np.bincount(ti, minlength=m), out=rp3[1:])
    out.append(("bulge", m, n, rp3.astype(np.int32), tj.astype(np.int32), synth.uniform_pm1(14, 0, np.arange(tj.size))))
    # 16 diagonals 1500 apart: their x windows do not fit the LDS budget of the staged DIA / HDC kernels, so the
    # direct kernels run (without and with scattered entries, which become the CSR remainder of HDC)
    spread = [1500 * k for k in range(-8, 8)]
    out.append(("spread16", *synth.banded_scatter(20000, spread, 0, 100, 15)))
    out.append(("spread16s", *synth.banded_scatter(20000, spread, 2, 100, 16)))
    # ten diagonals 600 apart on a matrix large enough for 512-thread DIA blocks: ten x windows per block in fp64, one
    # wide window in fp32 (two rows per lane); with scattered entries, HDC adds its remainder
    ten = [600 * k for k in range(-5, 5)]
    out.append(("spread10", *synth.banded_scatter(140000, ten, 0, 100, 21)))
    out.append(("spread10s", *synth.banded_scatter(140000, ten, 2, 100, 22)))
    # a band with as many scattered entries as the feature traversal's candidate lists do not survive (30 %): the band's
    # diagonals are then counted entry by entry through the block's table of frequent diagonals
    out.append(("band30s", *synth.banded_scatter(60000, synth.C4_OFFSETS, 30, 100, 17)))
    # a band of 40 diagonals: every row is longer than the traversal's lane-per-row limit and is walked by a whole wave
    out.append(("band40", *synth.banded_scatter(20000, range(-20, 20), 1, 100, 18)))
    return out


CASES = small_cases()
IDS = [c[0] for c in CASES]


@pytest.mark.parametrize("case", CASES, ids=IDS)
def test_features_bit_exact(case):
    name, m, n, rp, ci, v = case
    a = upload(m, n, rp, ci, v)
    ti, tj, _ = ref.csr_to_triplets(rp, ci, v)
    for td in ((1, 2), (1, 16)):
        f, ints = mo.mo_features(a, dict(td_num=td[0], td_den=td[1]))
        fo, io = ref.features(m, n, ti, tj, td)
        assert f.tobytes() == fo.tobytes(), (f, fo)
        assert ints == io


def check_arrays(name, e, m, n, ti, tj, ta, params, hyb=(1, 3), td=(1, 2)):
    fmt = e["fmt"]
    if fmt == mo.MO_COO:
        r, c, v = ref.to_coo(ti, tj, ta)
        assert np.array_equal(e["coo_row"], r) and np.array_equal(e["coo_col"], c)
        assert e["coo_val"].astype(np.float64).tobytes() == v.tobytes()
    if fmt == mo.MO_DIA:
        off, val = ref.to_dia(m, n, ti, tj, ta)
        assert e["nd"] == off.shape[0] and np.array_equal(e["dia_off"], off)
        assert e["dia_val"][:, :m].astype(np.float64).tobytes() == val.tobytes()
    if fmt == mo.MO_ELL:
        k, col, val = ref.to_ell(m, ti, tj, ta)
        assert e["k"] == k
        assert np.array_equal(e["ell_col"][:, :m], col)
        assert e["ell_val"][:, :m].astype(np.float64).tobytes() == val.tobytes()
    if fmt == mo.MO_HYB:
        h = ref.to_hyb(m, ti, tj, ta, hyb)
        assert e["k"] == h["k"] and e["nnz_coo"] == h["coo_row"].shape[0]
        assert np.array_equal(e["ell_col"][:, :m], h["ell_col"])
        assert e["ell_val"][:, :m].astype(np.float64).tobytes() == h["ell_val"].tobytes()
        assert np.array_equal(e["coo_row"], h["coo_row"]) and np.array_equal(e["coo_col"], h["coo_col"])
        assert e["coo_val"].astype(np.float64).tobytes() == h["coo_val"].tobytes()
    if fmt == mo.MO_HDC:
        h = ref.to_hdc(m, n, ti, tj, ta, td)
        assert e["nd"] == h["dia_off"].shape[0] and np.array_equal(e["dia_off"], h["dia_off"])
        assert e["dia_val"][:, :m].astype(np.float64).tobytes() == h["dia_val"].tobytes()
        assert np.array_equal(e["csr_row_ptr"], h["csr_row_ptr"]) and np.array_equal(e["csr_col"], h["csr_col"])
        assert e["csr_val"].astype(np.float64).tobytes() == h["csr_val"].tobytes()
        assert e["nnz_csr"] == h["csr_col"].shape[0]
    if fmt == mo.MO_CSR:
        wrp, wc, wv = ref.to_csr(m, ti, tj, ta)
        assert np.array_equal(e["csr_row_ptr"], wrp) and np.array_equal(e["csr_col"], wc)
        assert e["csr_val"].astype(np.float64).tobytes() == wv.tobytes()
        assert np.array_equal(wrp, rp_of(ti, m))


def rp_of(ti, m):
    rp = np.zeros(m + 1, np.int64)
    np.cumsum(np.bincount(ti, minlength=m), out=rp[1:])
    return rp.astype(np.int32)


def oracle_feasible(fmt, m, n, ti, tj, max_fill=16):
    nnz = ti.shape[0]
    if fmt == mo.MO_DIA:
        f, _ = ref.features(m, n, ti, tj)
        return ref.feasible(int(f[8]) * m, nnz, max_fill)
    if fmt == mo.MO_ELL:
        return ref.feasible(ref.max_row(m, ti) * m, nnz, max_fill)
    return True


@pytest.mark.parametrize("dtype", [np.float64, np.float32], ids=["f64", "f32"])
@pytest.mark.parametrize("case", CASES, ids=IDS)
def test_convert_and_spmv(case, dtype):
    name, m, n, rp, ci, v = case
    a = upload(m, n, rp, ci, v, dtype)
    x = synth.make_x(n, 3)
    ti, tj, ta, xo = oracle_inputs(rp, ci, v, x, dtype)
    y_ref, mag = ref.spmv(m, n, ti, tj, ta, xo)
    # a looser padding limit than the default so that DIA / ELL are exercised on more of the small cases
    params = dict(max_fill=256)
    ys = {}
    for fmt in range(6):
        h = try_convert(a, fmt, params)
        assert (h is not None) == oracle_feasible(fmt, m, n, ti, tj, 256), mo.FORMAT_NAMES[fmt]
        if h is None:
            continue
        e = h.export()
        assert (e["m"], e["n"], e["nnz"], e["fmt"]) == (m, n, rp[-1], fmt)
        check_arrays(name, e, m, n, ti, tj, ta, params)
        y = gpu_spmv(h, x, m, dtype)
        err, zeros_ok = ref.spmv_error(y, y_ref, mag)
        assert err <= TOL[dtype], (mo.FORMAT_NAMES[fmt], err)
        assert zeros_ok, mo.FORMAT_NAMES[fmt]
        # bit-identical on a second run (no floating-point atomics anywhere)
        assert gpu_spmv(h, x, m, dtype).tobytes() == y.tobytes()
        ys[fmt] = y.astype(np.float64)
        h.free()
    for fmt in ys:
        nz = mag > 0
        if nz.any():
            assert np.max(np.abs(ys[fmt][nz] - ys[mo.MO_CSR][nz]) / mag[nz]) <= 2 * TOL[dtype]


@pytest.mark.parametrize("dtype", [np.float64, np.float32], ids=["f64", "f32"])
@pytest.mark.parametrize("scatter", [0, 2], ids=["dia", "hdc"])
def test_batched_dia_kernel(scatter, dtype):
    """Half a million rows (plus a ragged tail) with ten diagonals 600 apart: the batched DIA / HDC kernel runs, and its
    x windows (fp64: ten of 512 positions; fp32, two rows per lane: one of 6424) exceed what a block requests in its first
    batch, so the staging loop runs a second one.  With scattered entries HDC adds its remainder through the 2-byte row
    offsets per row block."""
    m, n, rp, ci, v = synth.banded_scatter((1 << 19) + 77, [600 * k for k in range(-5, 5)], scatter, 100, 24)
    a = upload(m, n, rp, ci, v, dtype)
    x = synth.make_x(n, 6)
    ti, tj, ta, xo = oracle_inputs(rp, ci, v, x, dtype)
    y_ref, mag = ref.spmv(m, n, ti, tj, ta, xo)
    for fmt in ((mo.MO_DIA, mo.MO_HDC) if scatter == 0 else (mo.MO_HDC,)):
        h = mo.mo_convert(a, fmt)
        assert h.kernels() == "k_dia_batch", h.kernels()
        y = gpu_spmv(h, x, m, dtype)
        err, zeros_ok = ref.spmv_error(y, y_ref, mag)
        assert err <= TOL[dtype] and zeros_ok, (mo.FORMAT_NAMES[fmt], err)
        assert gpu_spmv(h, x, m, dtype).tobytes() == y.tobytes()
        if fmt == mo.MO_HDC and scatter:
            e = h.export()
            assert e["nnz_csr"] > 0 and e["nd"] == 10
            hd = ref.to_hdc(m, n, ti, tj, ta)
            assert np.array_equal(e["csr_row_ptr"], hd["csr_row_ptr"]) and np.array_equal(e["csr_col"], hd["csr_col"])
        h.free()


@pytest.mark.parametrize("offsets", [[0], [-2, -1, 0, 1], [-3000, -2, -1, 0, 1, 2, 3000], [700 * k for k in range(-6, 6)]],
                         ids=["nd1", "nd4", "nd7", "nd12"])
def test_batched_dia_kernel_by_number_of_diagonals(offsets):
    """The batched kernel is instantiated per number of diagonals (1 .. 12): one diagonal, one window of four, three
    windows of seven, twelve windows of twelve, each as HDC with 1 % scattered entries in fp64 and as DIA / HDC without
    them in fp32 (where the twelve merge into one window that is too long for the batched kernel's plan)."""
    for scatter, dtype in ((1, np.float64), (0, np.float32)):
        m, n, rp, ci, v = synth.banded_scatter((1 << 19) + 5, offsets, scatter, 100, 25 + len(offsets))
        a = upload(m, n, rp, ci, v, dtype)
        x = synth.make_x(n, 7)
        ti, tj, ta, xo = oracle_inputs(rp, ci, v, x, dtype)
        y_ref, mag = ref.spmv(m, n, ti, tj, ta, xo)
        for fmt in ((mo.MO_HDC,) if scatter else (mo.MO_DIA, mo.MO_HDC)):
            h = mo.mo_convert(a, fmt)
            # twelve diagonals 700 apart in fp32 (two rows per lane: blocks of 1024 rows) merge into one window of 8724
            # positions, more than the plan in the kernel arguments holds: the streaming kernel runs
            want = "k_dia_lds" if len(offsets) == 12 and dtype == np.float32 else "k_dia_batch"
            assert h.kernels() == want and h.view().nd == len(offsets), (h.kernels(), h.view().nd)
            y = gpu_spmv(h, x, m, dtype)
            err, zeros_ok = ref.spmv_error(y, y_ref, mag)
            assert err <= TOL[dtype] and zeros_ok, (mo.FORMAT_NAMES[fmt], len(offsets), err)
            h.free()


@pytest.mark.parametrize("m,dtype,skewed", [(1 << 16, np.float64, True), (1 << 16, np.float32, True), ((1 << 16) + 64, np.float64, False),
                                            (1 << 13, np.float32, False)], ids=["2^16-f64", "2^16-f32", "2^16+64-f64", "2^13-f32"])
def test_slab_stride_off_powers_of_two(m, dtype, skewed):
    """Slabs that would lie a multiple of 64 KB apart get 576 rows more each (the exported ld says so), every other
    matrix keeps ld = M rounded up to 64; the arrays over [:, :m] and the product are the oracle's either way."""
    mm, n, rp, ci, v = synth.banded_scatter(m, [-1, 0, 1], 0, 100, 31)
    a = upload(mm, n, rp, ci, v, dtype)
    x = synth.make_x(n, 8)
    ti, tj, ta, xo = oracle_inputs(rp, ci, v, x, dtype)
    y_ref, mag = ref.spmv(mm, n, ti, tj, ta, xo)
    for fmt in (mo.MO_DIA, mo.MO_ELL):
        h = mo.mo_convert(a, fmt)
        e = h.export()
        assert e["ld"] == (mm + 63) // 64 * 64 + (576 if skewed else 0), e["ld"]
        check_arrays("stride", e, mm, n, ti, tj, ta, None)
        err, zeros_ok = ref.spmv_error(gpu_spmv(h, x, mm, dtype), y_ref, mag)
        assert err <= TOL[dtype] and zeros_ok, (mo.FORMAT_NAMES[fmt], err)
        h.free()


@pytest.mark.parametrize("scatter", [0, 1], ids=["ell", "hyb"])
def test_ell_windows_in_two_batches(scatter):
    """Eight groups of four neighbouring diagonals on 320 000 rows: the ELL / HYB kernel with x windows stages 8 x 515
    positions per block of 512 rows, more than its first batch of requests holds.  A few scattered entries give HYB a
    COO part whose first entry per row travels with the slots."""
    offs = [3000 * g + d for g in range(-4, 4) for d in range(4)]
    m, n, rp, ci, v = synth.banded_scatter(320000, offs, scatter, 100, 23)
    a = upload(m, n, rp, ci, v)
    x = synth.make_x(n, 5)
    ti, tj, ta, xo = oracle_inputs(rp, ci, v, x, np.float64)
    y_ref, mag = ref.spmv(m, n, ti, tj, ta, xo)
    for fmt in (mo.MO_ELL, mo.MO_HYB):
        h = mo.mo_convert(a, fmt, dict(max_fill=256))
        assert h.kernels().startswith("k_ell_win"), h.kernels()
        y = gpu_spmv(h, x, m, np.float64)
        err, zeros_ok = ref.spmv_error(y, y_ref, mag)
        assert err <= TOL[np.float64] and zeros_ok, (mo.FORMAT_NAMES[fmt], err)
        assert gpu_spmv(h, x, m, np.float64).tobytes() == y.tobytes()
        h.free()


@pytest.mark.parametrize("case", CASES, ids=IDS)
def test_default_fill_limit_matches_oracle(case):
    name, m, n, rp, ci, v = case
    a = upload(m, n, rp, ci, v)
    ti, tj, _ = ref.csr_to_triplets(rp, ci, v)
    for fmt in (mo.MO_DIA, mo.MO_ELL):
        h = try_convert(a, fmt)
        assert (h is not None) == oracle_feasible(fmt, m, n, ti, tj), mo.FORMAT_NAMES[fmt]
        if h is not None:
            h.free()


@pytest.mark.parametrize("params,hyb,td", [(dict(hyb_num=1, hyb_den=2, td_num=1, td_den=8), (1, 2), (1, 8)),
                                            (dict(hyb_num=0, hyb_den=1, td_num=1, td_den=1), (0, 1), (1, 1)),
                                            (dict(hyb_num=3, hyb_den=2, td_num=0, td_den=1), (3, 2), (0, 1))])
@pytest.mark.parametrize("cname", ["c3s", "c4s", "rect_wide"])
def test_hybrid_parameters(cname, params, hyb, td):
    name, m, n, rp, ci, v = CASES[IDS.index(cname)]
    a = upload(m, n, rp, ci, v)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    x = synth.make_x(n, 4)
    y_ref, mag = ref.spmv(m, n, ti, tj, ta, x)
    for fmt in (mo.MO_HYB, mo.MO_HDC):
        h = mo.mo_convert(a, fmt, params)
        check_arrays(name, h.export(), m, n, ti, tj, ta, params, hyb, td)
        err, zeros_ok = ref.spmv_error(gpu_spmv(h, x, m, np.float64), y_ref, mag)
        assert err <= 1e-13 and zeros_ok
        h.free()


def test_c1_unit_vector_and_ones():
    m, n, rp, ci, v = synth.config(1)
    a = upload(m, n, rp, ci, v)
    for fmt in range(6):
        h = mo.mo_convert(a, fmt)
        y = gpu_spmv(h, np.ones(n), m, np.float64)
        r = np.arange(m)
        nb = (r % 64 == 0).astype(int) + (r % 64 == 63) + (r // 64 == 0) + (r // 64 == 63)
        assert np.array_equal(y, nb.astype(np.float64))
        e = np.zeros(n)
        e[1000] = 1.0
        y = gpu_spmv(h, e, m, np.float64)
        want = np.zeros(m)
        want[[1000 - 64, 999, 1000, 1001, 1064]] = [-1, -1, 4, -1, -1]
        assert np.array_equal(y, want)
        h.free()


def bad_csr(kind):
    m, n, rp, ci, v = synth.random_csr(200, 150, 0.1, 21)
    rp, ci = rp.copy(), ci.copy()
    if kind == "rp0":
        rp[0] = 1
    elif kind == "rp_decreasing":
        rp[50], rp[51] = rp[51] + 3, rp[50]
    elif kind == "rp_last":
        rp[-1] -= 1
    elif kind == "rp_beyond":
        rp[100] = rp[-1] + 1000
    elif kind == "rp_negative":
        rp[10] = -5
    elif kind == "col_high":
        ci[37] = n
    elif kind == "col_negative":
        ci[37] = -1
    elif kind == "col_unsorted":
        p = int(np.nonzero(np.diff(rp) >= 2)[0][0])
        s = rp[p]
        ci[s], ci[s + 1] = ci[s + 1], ci[s]
    elif kind == "col_duplicate":
        p = int(np.nonzero(np.diff(rp) >= 2)[0][0])
        ci[rp[p] + 1] = ci[rp[p]]
    elif kind in ("vlong_unsorted", "vlong_col_high"):
        m, n, rp, ci, v = very_long_rows()
        ci = ci.copy()
        if kind == "vlong_unsorted":
            ci[rp[20001] + 7000], ci[rp[20001] + 7001] = ci[rp[20001] + 7001], ci[rp[20001] + 7000]
        else:
            ci[rp[701] - 1] = n
    elif kind == "long_row_unsorted":
        m, n, rp, ci, v = synth.random_csr(4, 400, 0.9, 22)
        ci = ci.copy()
        ci[rp[2] + 200], ci[rp[2] + 201] = ci[rp[2] + 201], ci[rp[2] + 200]
    return m, n, rp, ci, v


@pytest.mark.parametrize("kind", ["rp0", "rp_decreasing", "rp_last", "rp_beyond", "rp_negative", "col_high", "col_negative",
                                  "col_unsorted", "col_duplicate", "long_row_unsorted", "vlong_unsorted", "vlong_col_high"])
def test_invalid_csr_is_rejected(kind):
    m, n, rp, ci, v = bad_csr(kind)
    a = upload(m, n, rp, ci, v)
    with pytest.raises(mo.MoError) as e:
        mo.mo_features(a)
    assert e.value.status == mo.MO_E_CSR_INVALID
    for fmt in range(6):
        with pytest.raises(mo.MoError) as e:
            mo.mo_convert(a, fmt)
        assert e.value.status == mo.MO_E_CSR_INVALID
    with pytest.raises(mo.MoError) as e:
        mo.mo_tune(a, reps=1, warmups=0)
    assert e.value.status == mo.MO_E_CSR_INVALID


@pytest.mark.parametrize("cname", ["c1", "c3s", "c4s", "empty"])
def test_tune_bookkeeping(cname):
    name, m, n, rp, ci, v = CASES[IDS.index(cname)]
    a = upload(m, n, rp, ci, v)
    ti, tj, _ = ref.csr_to_triplets(rp, ci, v)
    best, ms, cv = mo.mo_tune(a, warmups=1, reps=3)
    for fmt in range(6):
        assert (not np.isnan(ms[fmt])) == oracle_feasible(fmt, m, n, ti, tj), mo.FORMAT_NAMES[fmt]
        assert np.isnan(ms[fmt]) == np.isnan(cv[fmt])
    assert best == ref.pick(ms) == mo.mo_pick(ms)
    assert np.all(ms[~np.isnan(ms)] > 0)


def test_other_stream_and_default_allocator():
    m, n, rp, ci, v = synth.config(2, 0.1)
    a = upload(m, n, rp, ci, v)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    x = synth.make_x(n, 9)
    y_ref, mag = ref.spmv(m, n, ti, tj, ta, x)
    s = torch.cuda.Stream()
    xd = torch.as_tensor(x).cuda()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        for fmt in range(6):
            h = mo.mo_convert(a, fmt, stream=s)
            y = torch.empty(m, dtype=torch.float64, device="cuda")
            mo.mo_spmv(h, xd, y, stream=s)
            s.synchronize()
            err, ok = ref.spmv_error(y.cpu().numpy(), y_ref, mag)
            assert err <= 1e-13 and ok
            h.free()


def test_features_scratch_is_reused_safely():
    """mo_features keeps its scratch between calls: growing and shrinking matrices, a rejected matrix in between, another
    stream and a change of allocator must all leave the next result exact."""
    seq = [("c1", None), ("c4s", None), ("tiny", None), ("bad", "col_high"), ("c2s", None), ("bad", "rp_decreasing"),
           ("rect_wide", None), ("c4s", None), ("empty", None), ("long_row", None)]
    other = torch.cuda.Stream()
    for step, (name, kind) in enumerate(seq):
        if name == "bad":
            a = upload(*bad_csr(kind))
            with pytest.raises(mo.MoError) as e:
                mo.mo_features(a)
            assert e.value.status == mo.MO_E_CSR_INVALID
            continue
        _, m, n, rp, ci, v = CASES[IDS.index(name)]
        a = upload(m, n, rp, ci, v)
        ti, tj, _ = ref.csr_to_triplets(rp, ci, v)
        fo, io = ref.features(m, n, ti, tj)
        if step == 6:       # back to hipMalloc / hipFree and on to torch's allocator again: the kept block is released
            assert mo.lib.mo_set_allocator(C.cast(None, mo._ALLOC_T), C.cast(None, mo._FREE_T), None) == mo.MO_OK
            f, ints = mo.mo_features(a)
            assert f.tobytes() == fo.tobytes() and ints == io
            assert mo.lib.mo_set_allocator(mo._alloc_cb, mo._free_cb, None) == mo.MO_OK
        for stream in (None, other):
            f, ints = mo.mo_features(a, stream=stream)
            assert f.tobytes() == fo.tobytes() and ints == io, (name, stream)


@pytest.mark.parametrize("dtype", [np.float64, np.float32], ids=["f64", "f32"])
def test_window_kernels_with_entries_outside_the_windows(dtype):
    """Matrices large enough for the kernels that serve x from LDS windows (ELL, fused HYB): a band of 15 diagonals plus
    two far ones, with 4 % scattered entries that fall outside every window (gathered from memory inside the same
    kernel), windows that reach past both ends of x, and a row count that is not a multiple of the block size."""
    m = 400003
    offs = list(range(-7, 8)) + [-30011, 25013]
    m, n, rp, ci, v = synth.banded_scatter(m, offs, 4, 100, 91)
    v = np.asarray(v, dtype=dtype)
    a = upload(m, n, rp, ci, v, dtype)
    x = synth.make_x(n, 92)
    ti, tj, ta, xo = oracle_inputs(rp, ci, v, x, dtype)
    y_ref, mag = ref.spmv(m, n, ti, tj, ta, xo)
    seen = set()
    for fmt in (mo.MO_ELL, mo.MO_HYB, mo.MO_CSR):
        h = try_convert(a, fmt, {"max_fill": 64})
        assert h is not None
        seen.add(h.kernels())
        y = gpu_spmv(h, x, m, dtype)
        err, zeros_ok = ref.spmv_error(y, y_ref, mag)
        assert err <= TOL[dtype] and zeros_ok, (mo.FORMAT_NAMES[fmt], err)
        assert gpu_spmv(h, x, m, dtype).tobytes() == y.tobytes()
        h.free()
    assert any("k_ell_win" in k for k in seen), seen


@pytest.mark.parametrize("rows,per_row,slices", [(1400000, 12, 2), (2800000, 6, 4), (1400000, 4, 0)], ids=["2-slices", "4-slices", "short-rows"])
def test_csr_column_slices_fp32(rows, per_row, slices):
    """Scattered columns and an x of 5.6 / 11.2 MB in fp32: the CSR handle multiplies in passes over 2 / 4 column slices
    (the fp64 case of that path is the lognormal configuration at full size); with rows too short for the passes to pay
    it stays with one pass."""
    m, n, rp, ci, v = synth.uniform_rows(rows, per_row, 93)
    v = np.asarray(v, dtype=np.float32)
    a = upload(m, n, rp, ci, v, np.float32)
    x = synth.make_x(n, 94)
    ti, tj, ta, xo = oracle_inputs(rp, ci, v, x, np.float32)
    y_ref, mag = ref.spmv(m, n, ti, tj, ta, xo)
    h = mo.mo_convert(a, mo.MO_CSR)
    assert h.kernels().startswith("%d column slices" % slices) if slices else "slices" not in h.kernels(), h.kernels()
    y = gpu_spmv(h, x, m, np.float32)
    err, zeros_ok = ref.spmv_error(y, y_ref, mag)
    assert err <= TOL[np.float32] and zeros_ok, err
    assert gpu_spmv(h, x, m, np.float32).tobytes() == y.tobytes()
    e = h.export()                                # the handle still exports the caller's CSR arrays
    assert np.array_equal(e["csr_row_ptr"], rp) and np.array_equal(e["csr_col"], ci) and e["csr_val"].tobytes() == v.tobytes()
    f, ints = mo.mo_matrix_features(h)
    fo, io = ref.features(m, n, ti, tj)
    assert f.tobytes() == fo.tobytes() and ints == io
    h.free()
