"""ctypes wrapper over the C oracle (test infrastructure only).

All functions take host numpy arrays.  The matrix is handed over as triplets
``(ti, tj, ta)``; ``csr_to_triplets`` expands the CSR arrays the GPU side
receives.  fp32 inputs are promoted exactly to fp64 first.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import build as _build

_lib = None

I32P = C.POINTER(C.c_int32)
I64P = C.POINTER(C.c_int64)
F64P = C.POINTER(C.c_double)
U8P = C.POINTER(C.c_uint8)

FMT_COO, FMT_CSR, FMT_DIA, FMT_ELL, FMT_HYB, FMT_HDC = range(6)


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build(force=False))
        _lib.orc_dia_offsets.restype = C.c_int64
        _lib.orc_max_row.restype = C.c_int64
        _lib.orc_hyb_k.restype = C.c_int64
        for name in ("orc_from_dia", "orc_from_ell", "orc_from_csr"):
            getattr(_lib, name).restype = C.c_int64
    return _lib


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a, t):
    return a.ctypes.data_as(t)


def _i64(v):
    return C.c_int64(int(v))


def csr_to_triplets(row_ptr, col_idx, val):
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    m = row_ptr.shape[0] - 1
    ti = np.repeat(np.arange(m, dtype=np.int32), np.diff(row_ptr))
    return ti, _i32(col_idx), _f64(val)


def spmv(m, n, ti, tj, ta, x):
    ti, tj, ta, x = _i32(ti), _i32(tj), _f64(ta), _f64(x)
    assert x.shape[0] == n
    y = np.zeros(max(m, 1), dtype=np.float64)
    mag = np.zeros(max(m, 1), dtype=np.float64)
    rc = lib().orc_spmv(_i64(m), _i64(n), _i64(ti.shape[0]), _p(ti, I32P), _p(tj, I32P), _p(ta, F64P),
                        _p(x, F64P), _p(y, F64P), _p(mag, F64P))
    if rc != 0:
        raise ValueError(f"orc_spmv failed: {rc}")
    return y[:m], mag[:m]


def spmm(m, n, ti, tj, ta, x):
    """Y = A X, X of shape (n, k) -> (Y, |A||X|), both (m, k)."""
    ti, tj, ta = _i32(ti), _i32(tj), _f64(ta)
    x = np.ascontiguousarray(x, dtype=np.float64)
    assert x.ndim == 2 and x.shape[0] == n
    k = x.shape[1]
    y = np.zeros((max(m, 1), k), dtype=np.float64)
    mag = np.zeros((max(m, 1), k), dtype=np.float64)
    rc = lib().orc_spmm(_i64(m), _i64(n), _i64(ti.shape[0]), _p(ti, I32P), _p(tj, I32P), _p(ta, F64P), _i64(k),
                        _p(x, F64P), _p(y, F64P), _p(mag, F64P))
    if rc != 0:
        raise ValueError(f"orc_spmm failed: {rc}")
    return y[:m], mag[:m]


def spmv_rowsorted_mt(m, ti, tj, ta, x, nthreads):
    ti, tj, ta, x = _i32(ti), _i32(tj), _f64(ta), _f64(x)
    y = np.zeros(max(m, 1), dtype=np.float64)
    rc = lib().orc_spmv_rowsorted_mt(_i64(m), _i64(ti.shape[0]), _p(ti, I32P), _p(tj, I32P), _p(ta, F64P),
                                     _p(x, F64P), _p(y, F64P), C.c_int(int(nthreads)))
    if rc != 0:
        raise ValueError(f"orc_spmv_rowsorted_mt failed: {rc}")
    return y[:m]


INT_NAMES = ("m", "n", "nnz", "max_row", "min_row", "n_diag", "n_true_diag", "sum_sq_row")


def features(m, n, ti, tj, td=(1, 2)):
    ti, tj = _i32(ti), _i32(tj)
    out = np.zeros(10, dtype=np.float64)
    ints = np.zeros(8, dtype=np.int64)
    rc = lib().orc_features(_i64(m), _i64(n), _i64(ti.shape[0]), _p(ti, I32P), _p(tj, I32P),
                            _i64(td[0]), _i64(td[1]), _p(out, F64P), _p(ints, I64P))
    if rc != 0:
        raise ValueError(f"orc_features failed: {rc}")
    return out, dict(zip(INT_NAMES, (int(v) for v in ints)))


def to_coo(ti, tj, ta):
    ti, tj, ta = _i32(ti), _i32(tj), _f64(ta)
    nnz = ti.shape[0]
    row = np.zeros(max(nnz, 1), np.int32)
    col = np.zeros(max(nnz, 1), np.int32)
    val = np.zeros(max(nnz, 1), np.float64)
    rc = lib().orc_to_coo(_i64(nnz), _p(ti, I32P), _p(tj, I32P), _p(ta, F64P), _p(row, I32P), _p(col, I32P), _p(val, F64P))
    assert rc == 0
    return row[:nnz], col[:nnz], val[:nnz]


def _dia_part(m, n, ti, tj, ta, all_nonempty, td):
    nnz = ti.shape[0]
    args = (_i64(m), _i64(n), _i64(nnz), _p(ti, I32P), _p(tj, I32P), C.c_int(1 if all_nonempty else 0),
            _i64(td[0]), _i64(td[1]))
    nd = int(lib().orc_dia_offsets(*args, None))
    assert nd >= 0
    off = np.zeros(max(nd, 1), np.int32)
    lib().orc_dia_offsets(*args, _p(off, I32P))
    val = np.zeros(max(nd * m, 1), np.float64)
    taken = np.zeros(max(nnz, 1), np.uint8)
    rc = lib().orc_fill_dia(_i64(m), _i64(n), _i64(nnz), _p(ti, I32P), _p(tj, I32P), _p(ta, F64P),
                            _i64(nd), _p(off, I32P), _p(val, F64P), _p(taken, U8P))
    assert rc == 0
    return off[:nd], val[:nd * m].reshape(nd, m), taken[:nnz]


def to_dia(m, n, ti, tj, ta):
    """-> (off int32[nd] ascending, val float64[nd, m])"""
    ti, tj, ta = _i32(ti), _i32(tj), _f64(ta)
    off, val, _ = _dia_part(m, n, ti, tj, ta, True, (1, 2))
    return off, val


def max_row(m, ti):
    ti = _i32(ti)
    return int(lib().orc_max_row(_i64(m), _i64(ti.shape[0]), _p(ti, I32P)))


def _ell_part(m, ti, tj, ta, k):
    nnz = ti.shape[0]
    col = np.zeros(max(k * m, 1), np.int32)
    val = np.zeros(max(k * m, 1), np.float64)
    rrow = np.zeros(max(nnz, 1), np.int32)
    rcol = np.zeros(max(nnz, 1), np.int32)
    rval = np.zeros(max(nnz, 1), np.float64)
    nrest = C.c_int64(0)
    rc = lib().orc_to_ell(_i64(m), _i64(nnz), _p(ti, I32P), _p(tj, I32P), _p(ta, F64P), _i64(k),
                          _p(col, I32P), _p(val, F64P), C.byref(nrest), _p(rrow, I32P), _p(rcol, I32P), _p(rval, F64P))
    assert rc == 0
    r = nrest.value
    return col[:k * m].reshape(k, m), val[:k * m].reshape(k, m), rrow[:r], rcol[:r], rval[:r]


def to_ell(m, ti, tj, ta):
    """-> (K, col int32[K, m], val float64[K, m]); K = max row length."""
    ti, tj, ta = _i32(ti), _i32(tj), _f64(ta)
    k = max_row(m, ti)
    col, val, rrow, _, _ = _ell_part(m, ti, tj, ta, k)
    assert rrow.shape[0] == 0
    return k, col, val


def hyb_k(m, ti, hyb=(1, 3)):
    ti = _i32(ti)
    return int(lib().orc_hyb_k(_i64(m), _i64(ti.shape[0]), _p(ti, I32P), _i64(hyb[0]), _i64(hyb[1])))


def to_hyb(m, ti, tj, ta, hyb=(1, 3)):
    ti, tj, ta = _i32(ti), _i32(tj), _f64(ta)
    k = hyb_k(m, ti, hyb)
    col, val, rrow, rcol, rval = _ell_part(m, ti, tj, ta, k)
    return dict(k=k, ell_col=col, ell_val=val, coo_row=rrow, coo_col=rcol, coo_val=rval)


def to_hdc(m, n, ti, tj, ta, td=(1, 2)):
    ti, tj, ta = _i32(ti), _i32(tj), _f64(ta)
    off, dval, taken = _dia_part(m, n, ti, tj, ta, False, td)
    nnz = ti.shape[0]
    nrest = int(nnz - taken.sum())
    row_ptr = np.zeros(m + 1, np.int32)
    col = np.zeros(max(nrest, 1), np.int32)
    val = np.zeros(max(nrest, 1), np.float64)
    tk = np.ascontiguousarray(taken if nnz else np.zeros(1, np.uint8))
    rc = lib().orc_rest_to_csr(_i64(m), _i64(nnz), _p(ti, I32P), _p(tj, I32P), _p(ta, F64P), _p(tk, U8P),
                               _p(row_ptr, I32P), _p(col, I32P), _p(val, F64P))
    assert rc == 0
    return dict(dia_off=off, dia_val=dval, csr_row_ptr=row_ptr, csr_col=col[:nrest], csr_val=val[:nrest])


def _trip_buffers(cnt):
    c = max(int(cnt), 1)
    return np.zeros(c, np.int32), np.zeros(c, np.int32), np.zeros(c, np.float64)


def from_dia(m, n, off, val):
    """DIA arrays (off[nd], val[nd, m]) -> triplets; exactly-zero and out-of-matrix positions are not entries."""
    off, val = _i32(off), _f64(val).reshape(-1)
    nd = off.shape[0]
    args = (_i64(m), _i64(n), _i64(nd), _p(off, I32P) if nd else None, _p(val, F64P) if val.size else None)
    cnt = int(lib().orc_from_dia(*args, None, None, None))
    ti, tj, ta = _trip_buffers(cnt)
    lib().orc_from_dia(*args, _p(ti, I32P), _p(tj, I32P), _p(ta, F64P))
    return ti[:cnt], tj[:cnt], ta[:cnt]


def from_ell(m, col, val):
    """ELL arrays (col[k, m], val[k, m]) -> triplets; slots with col >= 0 are entries."""
    k = col.shape[0]
    col, val = _i32(col).reshape(-1), _f64(val).reshape(-1)
    args = (_i64(m), _i64(k), _p(col, I32P) if col.size else None, _p(val, F64P) if val.size else None)
    cnt = int(lib().orc_from_ell(*args, None, None, None))
    ti, tj, ta = _trip_buffers(cnt)
    lib().orc_from_ell(*args, _p(ti, I32P), _p(tj, I32P), _p(ta, F64P))
    return ti[:cnt], tj[:cnt], ta[:cnt]


def from_csr(m, row_ptr, col, val):
    row_ptr, col, val = _i32(row_ptr), _i32(col), _f64(val)
    cnt = int(row_ptr[m])
    ti, tj, ta = _trip_buffers(cnt)
    got = int(lib().orc_from_csr(_i64(m), _p(row_ptr, I32P), _p(col, I32P) if cnt else None, _p(val, F64P) if cnt else None,
                                 _p(ti, I32P), _p(tj, I32P), _p(ta, F64P)))
    assert got == cnt
    return ti[:cnt], tj[:cnt], ta[:cnt]


def to_csr(m, ti, tj, ta):
    """-> (row_ptr int32[m+1], col int32[nnz], val float64[nnz]), columns ascending inside a row."""
    ti, tj, ta = _i32(ti), _i32(tj), _f64(ta)
    nnz = ti.shape[0]
    row_ptr = np.zeros(m + 1, np.int32)
    col, _, val = _trip_buffers(nnz)
    rc = lib().orc_to_csr(_i64(m), _i64(nnz), _p(ti, I32P), _p(tj, I32P), _p(ta, F64P), _p(row_ptr, I32P), _p(col, I32P), _p(val, F64P))
    assert rc == 0
    return row_ptr, col[:nnz], val[:nnz]


def format_to_triplets(fmt, m, n, arrays):
    """Triplets held by a matrix in format ``fmt`` given the oracle-layout arrays of that format (dict)."""
    parts = []
    if fmt in (FMT_DIA, FMT_HDC):
        parts.append(from_dia(m, n, arrays["dia_off"], arrays["dia_val"]))
    if fmt in (FMT_ELL, FMT_HYB):
        parts.append(from_ell(m, arrays["ell_col"], arrays["ell_val"]))
    if fmt in (FMT_COO, FMT_HYB):
        parts.append((_i32(arrays["coo_row"]), _i32(arrays["coo_col"]), _f64(arrays["coo_val"])))
    if fmt in (FMT_CSR, FMT_HDC):
        parts.append(from_csr(m, arrays["csr_row_ptr"], arrays["csr_col"], arrays["csr_val"]))
    return (np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts]), np.concatenate([p[2] for p in parts]))


def feasible(slots, nnz, max_fill=16, max_slots=(1 << 62)):
    return bool(lib().orc_feasible(_i64(slots), _i64(nnz), _i64(max_fill), _i64(max_slots)))


def select(model, x):
    """model: dict(tree_off, feature, threshold, left, right, klass, n_classes)."""
    tree_off = _i32(model["tree_off"])
    feat, thr = _i32(model["feature"]), _f64(model["threshold"])
    left, right, klass = _i32(model["left"]), _i32(model["right"]), _i32(model["klass"])
    x = _f64(x)
    return int(lib().orc_select(C.c_int32(tree_off.shape[0] - 1), _p(tree_off, I32P), _p(feat, I32P), _p(thr, F64P),
                                _p(left, I32P), _p(right, I32P), _p(klass, I32P),
                                C.c_int32(int(model.get("n_classes", 6))), _p(x, F64P)))


def pick(ms):
    ms = _f64(ms)
    return int(lib().orc_pick(C.c_int32(ms.shape[0]), _p(ms, F64P)))


def spmv_error(y_test, y_ref, mag):
    """max_i |y_test - y_ref|_i / mag_i over rows with mag_i > 0, and whether all
    rows with mag_i == 0 are exactly zero."""
    y_test = np.asarray(y_test, dtype=np.float64)
    nz = mag > 0
    err = float(np.max(np.abs(y_test[nz] - y_ref[nz]) / mag[nz])) if nz.any() else 0.0
    zeros_ok = bool(np.all(y_test[~nz] == 0.0))
    return err, zeros_ok
