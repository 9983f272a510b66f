"""Thin ctypes binding over ``libmo.so`` (the C ABI declared in ``include/mo.h``).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory (tensors, and the caching allocator
the library is pointed at) and streams.  There is no CPU fallback: if the
library has not been built, importing this module raises.

torch is imported before the library is loaded so that both share one HIP
runtime (the first ``libamdhip64.so.7`` in the process wins).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  (must precede the CDLL below)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmo.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2303_05098_amd.build` (or __graft_entry__.build()) first")

lib = C.CDLL(LIB_PATH)

MO_COO, MO_CSR, MO_DIA, MO_ELL, MO_HYB, MO_HDC = range(6)
FORMAT_NAMES = ("COO", "CSR", "DIA", "ELL", "HYB", "HDC")
MO_F32, MO_F64 = 0, 1
(MO_OK, MO_E_NULL, MO_E_SHAPE, MO_E_CSR_INVALID, MO_E_FORMAT, MO_E_DTYPE, MO_E_FILL, MO_E_ALLOC, MO_E_DEVICE,
 MO_E_MODEL, MO_E_PARAM, MO_E_IO) = range(12)

EXPORTS = ("mo_default_params", "mo_features", "mo_features_finalize", "mo_features_static", "mo_convert", "mo_spmv", "mo_spmv_kernels", "mo_spmm", "mo_tune", "mo_tune_spmm", "mo_pick", "mo_model_load",
           "mo_model_free", "mo_model_info", "mo_select", "mo_default_fit_opts", "mo_model_fit", "mo_model_save", "mo_predict", "mo_mtx_read", "mo_host_free", "mo_switch", "mo_matrix_features", "mo_matrix_export", "mo_matrix_free", "mo_set_allocator",
           "mo_strerror", "mo_last_hip_error")


class MoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.mo_strerror(status).decode()
        extra = f" (hipError {lib.mo_last_hip_error()})" if status == MO_E_DEVICE else ""
        super().__init__(f"{where}: {msg}{extra}")


class mo_csr(C.Structure):
    _fields_ = [("m", C.c_int64), ("n", C.c_int64), ("nnz", C.c_int64), ("row_ptr", C.c_void_p), ("col_idx", C.c_void_p),
                ("val", C.c_void_p), ("dtype", C.c_int)]


class mo_params(C.Structure):
    _fields_ = [("td_num", C.c_int32), ("td_den", C.c_int32), ("hyb_num", C.c_int32), ("hyb_den", C.c_int32),
                ("max_fill", C.c_int32), ("max_slots", C.c_int64)]


class mo_feature_ints(C.Structure):
    _fields_ = [("m", C.c_int64), ("n", C.c_int64), ("nnz", C.c_int64), ("max_row", C.c_int64), ("min_row", C.c_int64),
                ("n_diag", C.c_int64), ("n_true_diag", C.c_int64), ("sum_sq_row", C.c_uint64)]


class mo_feature_result(C.Structure):
    _fields_ = [("ints", mo_feature_ints), ("status", C.c_int32), ("pad", C.c_int32)]


class mo_tune_opts(C.Structure):
    _fields_ = [("warmups", C.c_int32), ("reps", C.c_int32)]


class mo_fit_opts(C.Structure):
    _fields_ = [("n_estimators", C.c_int32), ("bootstrap", C.c_int32), ("max_depth", C.c_int32),
                ("min_samples_leaf", C.c_int32), ("min_samples_split", C.c_int32), ("max_features", C.c_int32),
                ("criterion", C.c_int32), ("seed", C.c_uint64)]


class mo_matrix_view(C.Structure):
    _fields_ = [("fmt", C.c_int), ("dtype", C.c_int), ("m", C.c_int64), ("n", C.c_int64), ("nnz", C.c_int64),
                ("ld", C.c_int64), ("nd", C.c_int64), ("k", C.c_int64), ("nnz_coo", C.c_int64), ("nnz_csr", C.c_int64),
                ("dia_off", C.c_void_p), ("ell_col", C.c_void_p), ("coo_row", C.c_void_p), ("coo_col", C.c_void_p),
                ("csr_row_ptr", C.c_void_p), ("csr_col", C.c_void_p),
                ("dia_val", C.c_void_p), ("ell_val", C.c_void_p), ("coo_val", C.c_void_p), ("csr_val", C.c_void_p)]


_ALLOC_T = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p)
_FREE_T = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p, C.c_void_p)

lib.mo_strerror.restype = C.c_char_p
lib.mo_strerror.argtypes = [C.c_int]
lib.mo_last_hip_error.restype = C.c_int
lib.mo_default_params.restype = None
lib.mo_default_params.argtypes = [C.POINTER(mo_params)]
lib.mo_features.argtypes = [C.POINTER(mo_csr), C.POINTER(mo_params), C.POINTER(C.c_double), C.POINTER(mo_feature_ints), C.c_void_p]
lib.mo_features_finalize.argtypes = [C.POINTER(mo_feature_ints), C.POINTER(C.c_double)]
lib.mo_features_static.argtypes = [C.POINTER(mo_csr), C.POINTER(mo_params), C.c_void_p, C.c_void_p]
lib.mo_convert.argtypes = [C.POINTER(mo_csr), C.c_int, C.POINTER(mo_params), C.POINTER(C.c_void_p), C.c_void_p]
lib.mo_switch.argtypes = [C.c_void_p, C.c_int, C.POINTER(mo_params), C.POINTER(C.c_void_p), C.c_void_p]
lib.mo_matrix_features.argtypes = [C.c_void_p, C.POINTER(mo_params), C.POINTER(C.c_double), C.POINTER(mo_feature_ints), C.c_void_p]
lib.mo_spmv.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
lib.mo_spmv_kernels.argtypes = [C.c_void_p, C.c_char_p, C.c_size_t]
lib.mo_spmm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
lib.mo_tune_spmm.argtypes = [C.POINTER(mo_csr), C.c_int32, C.POINTER(mo_params), C.POINTER(mo_tune_opts), C.POINTER(C.c_int),
                             C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_void_p]
lib.mo_tune.argtypes = [C.POINTER(mo_csr), C.POINTER(mo_params), C.POINTER(mo_tune_opts), C.POINTER(C.c_int),
                        C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_void_p]
lib.mo_pick.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int)]
lib.mo_model_load.argtypes = [C.c_char_p, C.POINTER(C.c_void_p)]
lib.mo_model_free.restype = None
lib.mo_model_free.argtypes = [C.c_void_p]
lib.mo_model_info.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
lib.mo_select.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int)]
lib.mo_default_fit_opts.restype = None
lib.mo_default_fit_opts.argtypes = [C.POINTER(mo_fit_opts)]
lib.mo_model_fit.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(mo_fit_opts), C.POINTER(C.c_void_p)]
lib.mo_model_save.argtypes = [C.c_void_p, C.c_char_p]
lib.mo_predict.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
lib.mo_mtx_read.argtypes = [C.c_char_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                            C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]
lib.mo_host_free.restype = None
lib.mo_host_free.argtypes = [C.c_void_p]
lib.mo_matrix_export.argtypes = [C.c_void_p, C.POINTER(mo_matrix_view)]
lib.mo_matrix_free.restype = None
lib.mo_matrix_free.argtypes = [C.c_void_p]
lib.mo_set_allocator.argtypes = [_ALLOC_T, _FREE_T, C.c_void_p]


# ------------------------------------------------------------------ torch-backed device allocator
def _torch_alloc(nbytes, stream, _user):
    try:
        return torch.cuda.caching_allocator_alloc(int(nbytes), torch.cuda.current_device(), int(stream or 0))
    except Exception:
        return None


def _torch_free(ptr, _stream, _user):
    if ptr:
        torch.cuda.caching_allocator_delete(int(ptr))


_alloc_cb = _ALLOC_T(_torch_alloc)
_free_cb = _FREE_T(_torch_free)
_allocator_installed = False


def use_torch_allocator() -> None:
    """Route the library's device allocations through torch's caching allocator."""
    global _allocator_installed
    if not _allocator_installed:
        _check(lib.mo_set_allocator(_alloc_cb, _free_cb, None), "mo_set_allocator")
        _allocator_installed = True


def _check(status: int, where: str) -> None:
    if status != MO_OK:
        raise MoError(status, where)


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


def _params(params):
    if params is None:
        return None
    p = mo_params()
    lib.mo_default_params(C.byref(p))
    for k, v in params.items():
        if not hasattr(p, k):
            raise KeyError(k)
        setattr(p, k, v)
    return C.byref(p)


class Csr:
    """CSR arrays resident on the GPU as torch tensors (int32 / int32 / float32|float64)."""

    def __init__(self, m, n, row_ptr, col_idx, val, device="cuda"):
        self.m, self.n = int(m), int(n)
        self.row_ptr = torch.as_tensor(np.ascontiguousarray(row_ptr, dtype=np.int32)).to(device) if not torch.is_tensor(row_ptr) else row_ptr
        self.col_idx = torch.as_tensor(np.ascontiguousarray(col_idx, dtype=np.int32)).to(device) if not torch.is_tensor(col_idx) else col_idx
        self.val = torch.as_tensor(np.ascontiguousarray(val)).to(device) if not torch.is_tensor(val) else val
        if self.row_ptr.dtype != torch.int32 or self.col_idx.dtype != torch.int32:
            raise ValueError("row_ptr and col_idx must be int32")
        if self.val.dtype not in (torch.float32, torch.float64):
            raise ValueError("val must be float32 or float64")
        for name, t in (("row_ptr", self.row_ptr), ("col_idx", self.col_idx), ("val", self.val)):
            if not t.is_contiguous() or t.dim() != 1:
                raise ValueError(f"{name} must be a contiguous 1-D tensor")
            if str(device).startswith("cuda") and not t.is_cuda:
                raise ValueError(f"{name} must live on the GPU")
        if self.row_ptr.numel() != self.m + 1:
            raise ValueError(f"row_ptr has {self.row_ptr.numel()} entries, m + 1 = {self.m + 1} are needed")
        if self.val.numel() != self.col_idx.numel():
            raise ValueError("val and col_idx differ in length")
        self.nnz = int(self.col_idx.numel())
        self.dtype = MO_F32 if self.val.dtype == torch.float32 else MO_F64

    def struct(self, nnz=None) -> mo_csr:
        return mo_csr(self.m, self.n, self.nnz if nnz is None else nnz, self.row_ptr.data_ptr(), self.col_idx.data_ptr() or None,
                      self.val.data_ptr() or None, self.dtype)


class _DevView:
    def __init__(self, ptr, count, np_dtype):
        self.__cuda_array_interface__ = {"shape": (count,), "typestr": np.dtype(np_dtype).str, "data": (int(ptr), False), "version": 2}


def _to_host(ptr, count, np_dtype) -> np.ndarray:
    if not ptr or count <= 0:
        return np.zeros(0, dtype=np_dtype)
    return torch.as_tensor(_DevView(ptr, count, np_dtype), device="cuda").cpu().numpy().copy()


class Matrix:
    """Owner of one ``mo_matrix*``; ``keep`` pins the tensors a CSR handle borrows."""

    def __init__(self, handle, keep=None):
        self.handle = handle
        self._keep = keep

    def dims(self):
        """(m, n, torch dtype) of the held matrix, read once from the handle."""
        if getattr(self, "_dims", None) is None:
            v = self.view()
            self._dims = (int(v.m), int(v.n), torch.float32 if v.dtype == MO_F32 else torch.float64)
        return self._dims

    def view(self) -> mo_matrix_view:
        v = mo_matrix_view()
        _check(lib.mo_matrix_export(self.handle, C.byref(v)), "mo_matrix_export")
        return v

    def export(self) -> dict:
        """Every array of the handle copied to host numpy; 2-D slabs as [width, ld]."""
        v = self.view()
        vt = np.float32 if v.dtype == MO_F32 else np.float64
        out = dict(fmt=v.fmt, dtype=v.dtype, m=v.m, n=v.n, nnz=v.nnz, ld=v.ld, nd=v.nd, k=v.k, nnz_coo=v.nnz_coo, nnz_csr=v.nnz_csr)
        if v.fmt in (MO_DIA, MO_HDC):
            out["dia_off"] = _to_host(v.dia_off, v.nd, np.int32)
            out["dia_val"] = _to_host(v.dia_val, v.nd * v.ld, vt).reshape(v.nd, v.ld)
        if v.fmt in (MO_ELL, MO_HYB):
            out["ell_col"] = _to_host(v.ell_col, v.k * v.ld, np.int32).reshape(v.k, v.ld)
            out["ell_val"] = _to_host(v.ell_val, v.k * v.ld, vt).reshape(v.k, v.ld)
        if v.fmt in (MO_COO, MO_HYB):
            out["coo_row"] = _to_host(v.coo_row, v.nnz_coo, np.int32)
            out["coo_col"] = _to_host(v.coo_col, v.nnz_coo, np.int32)
            out["coo_val"] = _to_host(v.coo_val, v.nnz_coo, vt)
        if v.fmt in (MO_CSR, MO_HDC):
            out["csr_row_ptr"] = _to_host(v.csr_row_ptr, v.m + 1, np.int32)
            out["csr_col"] = _to_host(v.csr_col, v.nnz_csr, np.int32)
            out["csr_val"] = _to_host(v.csr_val, v.nnz_csr, vt)
        return out

    def kernels(self) -> str:
        """Names of the kernels mo_spmv launches for this handle."""
        buf = C.create_string_buffer(256)
        _check(lib.mo_spmv_kernels(self.handle, buf, 256), "mo_spmv_kernels")
        return buf.value.decode()

    def free(self) -> None:
        if self.handle:
            lib.mo_matrix_free(self.handle)
            self.handle = None
            self._keep = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


# ------------------------------------------------------------------ the C-ABI calls, same names
def mo_features(a: Csr, params=None, stream=None):
    """-> (features float64[10], ints dict)"""
    out = (C.c_double * 10)()
    ints = mo_feature_ints()
    st = a.struct()
    _check(lib.mo_features(C.byref(st), _params(params), out, C.byref(ints), _stream_ptr(stream)), "mo_features")
    return np.array(list(out), dtype=np.float64), {k: int(getattr(ints, k)) for k, _ in mo_feature_ints._fields_}


def mo_features_finalize(ints: dict) -> np.ndarray:
    """The ten doubles of Table I from the integer statistics (host only)."""
    st = mo_feature_ints(**{k: int(ints[k]) for k, _ in mo_feature_ints._fields_})
    out = (C.c_double * 10)()
    _check(lib.mo_features_finalize(C.byref(st), out), "mo_features_finalize")
    return np.array(list(out), dtype=np.float64)


STATIC_MAX_DIAGS = 4194304
RESULT_BYTES = C.sizeof(mo_feature_result)


def mo_features_static(a: Csr, out_dev: torch.Tensor, params=None, stream=None) -> None:
    """Enqueue the feature kernels without allocating or synchronising; ``out_dev``: a CUDA uint8 tensor of at least
    RESULT_BYTES bytes that receives a ``mo_feature_result``.  Decode it with ``decode_feature_result`` once the stream
    has finished."""
    if not (out_dev.is_cuda and out_dev.is_contiguous() and out_dev.dtype == torch.uint8 and out_dev.numel() >= RESULT_BYTES):
        raise ValueError(f"out_dev must be a contiguous CUDA uint8 tensor of at least {RESULT_BYTES} bytes")
    st = a.struct()
    _check(lib.mo_features_static(C.byref(st), _params(params), out_dev.data_ptr(), _stream_ptr(stream)), "mo_features_static")


def decode_feature_result(host_bytes) -> tuple:
    """bytes of a mo_feature_result -> (status, ints dict)"""
    r = mo_feature_result.from_buffer_copy(bytes(host_bytes)[:RESULT_BYTES])
    return int(r.status), {k: int(getattr(r.ints, k)) for k, _ in mo_feature_ints._fields_}


def mo_convert(a: Csr, fmt: int, params=None, stream=None) -> Matrix:
    h = C.c_void_p()
    st = a.struct()
    _check(lib.mo_convert(C.byref(st), int(fmt), _params(params), C.byref(h), _stream_ptr(stream)), "mo_convert")
    return Matrix(h, keep=a if fmt == MO_CSR else None)


def mo_switch(a: Matrix, fmt: int, params=None, stream=None) -> Matrix:
    h = C.c_void_p()
    _check(lib.mo_switch(a.handle, int(fmt), _params(params), C.byref(h), _stream_ptr(stream)), "mo_switch")
    return Matrix(h)


def mo_matrix_features(a: Matrix, params=None, stream=None):
    """-> (features float64[10], ints dict) of a matrix in whatever format the handle holds"""
    out = (C.c_double * 10)()
    ints = mo_feature_ints()
    _check(lib.mo_matrix_features(a.handle, _params(params), out, C.byref(ints), _stream_ptr(stream)), "mo_matrix_features")
    return np.array(list(out), dtype=np.float64), {k: int(getattr(ints, k)) for k, _ in mo_feature_ints._fields_}


def _check_operands(a: Matrix, x, y, k: int, where: str) -> None:
    """The kernels trust the pointers they are given: refuse on the host whatever would make them read or write outside
    x or y (wrong device, dtype, length or layout)."""
    if not a.handle:
        raise ValueError(f"{where}: the matrix handle has been freed")
    m, n, dt = a.dims()
    for name, t, need in (("x", x, n * k), ("y", y, m * k)):
        if not torch.is_tensor(t) or not t.is_cuda:
            raise ValueError(f"{where}: {name} must be a CUDA tensor")
        if t.dtype != dt:
            raise ValueError(f"{where}: {name} is {t.dtype}, the matrix holds {dt}")
        if not t.is_contiguous():
            raise ValueError(f"{where}: {name} must be contiguous")
        if t.numel() < need:
            raise ValueError(f"{where}: {name} has {t.numel()} elements, {need} are needed")


def mo_spmv(a: Matrix, x: torch.Tensor, y: torch.Tensor, stream=None) -> None:
    _check_operands(a, x, y, 1, "mo_spmv")
    _check(lib.mo_spmv(a.handle, x.data_ptr(), y.data_ptr(), _stream_ptr(stream)), "mo_spmv")


def mo_tune(a: Csr, params=None, warmups=5, reps=50, stream=None):
    """-> (best format id, ms_per_rep float64[6] (NaN = infeasible), convert_ms float64[6])"""
    best = C.c_int(-1)
    ms = (C.c_double * 6)()
    cv = (C.c_double * 6)()
    opts = mo_tune_opts(int(warmups), int(reps))
    st = a.struct()
    _check(lib.mo_tune(C.byref(st), _params(params), C.byref(opts), C.byref(best), ms, cv, _stream_ptr(stream)), "mo_tune")
    return best.value, np.array(list(ms)), np.array(list(cv))


def mo_spmm(a: Matrix, x: torch.Tensor, y: torch.Tensor, stream=None) -> None:
    """Y = A X; x: (n, k) and y: (m, k) contiguous row-major tensors of the handle's dtype."""
    if x.dim() != 2 or y.dim() != 2 or x.shape[1] != y.shape[1] or not x.is_contiguous() or not y.is_contiguous():
        raise ValueError("x must be (n, k) and y (m, k), both contiguous")
    _check_operands(a, x, y, int(x.shape[1]), "mo_spmm")
    _check(lib.mo_spmm(a.handle, x.data_ptr(), y.data_ptr(), int(x.shape[1]), _stream_ptr(stream)), "mo_spmm")


def mo_tune_spmm(a: Csr, k: int, params=None, warmups=5, reps=50, stream=None):
    """mo_tune with the k-vector product timed in place of SpMV."""
    best = C.c_int(-1)
    ms = (C.c_double * 6)()
    cv = (C.c_double * 6)()
    opts = mo_tune_opts(int(warmups), int(reps))
    st = a.struct()
    _check(lib.mo_tune_spmm(C.byref(st), int(k), _params(params), C.byref(opts), C.byref(best), ms, cv, _stream_ptr(stream)), "mo_tune_spmm")
    return best.value, np.array(list(ms)), np.array(list(cv))


def mo_pick(ms) -> int:
    arr = (C.c_double * 6)(*[float(v) for v in ms])
    best = C.c_int(-1)
    _check(lib.mo_pick(arr, C.byref(best)), "mo_pick")
    return best.value


class Model:
    def __init__(self, handle):
        self.handle = handle

    def info(self):
        nt, nn = C.c_int32(), C.c_int32()
        _check(lib.mo_model_info(self.handle, C.byref(nt), C.byref(nn)), "mo_model_info")
        return nt.value, nn.value

    def free(self):
        if self.handle:
            lib.mo_model_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def mo_model_load(path: str) -> Model:
    h = C.c_void_p()
    _check(lib.mo_model_load(os.fsencode(path), C.byref(h)), "mo_model_load")
    return Model(h)


def mo_select(model: Model, features) -> int:
    arr = (C.c_double * 10)(*[float(v) for v in features])
    out = C.c_int(-1)
    _check(lib.mo_select(model.handle, arr, C.byref(out)), "mo_select")
    return out.value


def mo_mtx_read(path: str):
    """Matrix Market file -> (m, n, row_ptr, col_idx, val) as numpy arrays on the host."""
    m, n, nnz = C.c_int64(), C.c_int64(), C.c_int64()
    rp, ci, va = C.c_void_p(), C.c_void_p(), C.c_void_p()
    _check(lib.mo_mtx_read(os.fsencode(path), C.byref(m), C.byref(n), C.byref(nnz), C.byref(rp), C.byref(ci), C.byref(va)), "mo_mtx_read")
    try:
        row_ptr = np.ctypeslib.as_array(C.cast(rp, C.POINTER(C.c_int32)), shape=(m.value + 1,)).copy()
        col_idx = np.ctypeslib.as_array(C.cast(ci, C.POINTER(C.c_int32)), shape=(max(nnz.value, 1),))[:nnz.value].copy()
        val = np.ctypeslib.as_array(C.cast(va, C.POINTER(C.c_double)), shape=(max(nnz.value, 1),))[:nnz.value].copy()
    finally:
        lib.mo_host_free(rp); lib.mo_host_free(ci); lib.mo_host_free(va)
    return m.value, n.value, row_ptr, col_idx, val


MO_GINI, MO_ENTROPY = 0, 1
CRITERIA = {"gini": MO_GINI, "entropy": MO_ENTROPY}


def fit_opts(**kw) -> mo_fit_opts:
    """The library's defaults (baseline column of Table III) with the given fields replaced."""
    o = mo_fit_opts()
    lib.mo_default_fit_opts(C.byref(o))
    for k, v in kw.items():
        if k == "criterion" and isinstance(v, str):
            v = CRITERIA[v]
        if not hasattr(o, k):
            raise TypeError(f"unknown training option {k}")
        setattr(o, k, int(v))
    return o


def mo_model_fit(X, y, **opts) -> Model:
    X = np.ascontiguousarray(X, dtype=np.float64)
    y = np.ascontiguousarray(y, dtype=np.int32)
    if X.ndim != 2 or X.shape[1] != 10 or y.shape != (X.shape[0],):
        raise ValueError("X must be n x 10 and y of length n")
    o = fit_opts(**opts)
    h = C.c_void_p()
    _check(lib.mo_model_fit(X.ctypes.data, y.ctypes.data, X.shape[0], C.byref(o), C.byref(h)), "mo_model_fit")
    return Model(h)


def mo_model_save(model: Model, path: str) -> None:
    _check(lib.mo_model_save(model.handle, os.fsencode(path)), "mo_model_save")


def mo_predict(model: Model, X) -> np.ndarray:
    X = np.ascontiguousarray(X, dtype=np.float64).reshape(-1, 10)
    out = np.empty(X.shape[0], dtype=np.int32)
    _check(lib.mo_predict(model.handle, X.ctypes.data, X.shape[0], out.ctypes.data), "mo_predict")
    return out


def read_model(path: str) -> list:
    """Parse a model file back into the list-of-dicts form write_model takes."""
    raw = open(path, "rb").read()
    if raw[:8] != b"MOMDL1\0\0":
        raise ValueError("not a model file")
    hdr = np.frombuffer(raw, dtype="<i4", count=4, offset=8)
    pos, trees = 24, []
    for _ in range(int(hdr[3])):
        nn = int(np.frombuffer(raw, dtype="<i4", count=1, offset=pos)[0])
        pos += 4
        t = {}
        for key, dt, sz in (("feature", "<i4", 4), ("threshold", "<f8", 8), ("left", "<i4", 4), ("right", "<i4", 4), ("klass", "<i4", 4)):
            t[key] = np.frombuffer(raw, dtype=dt, count=nn, offset=pos).tolist()
            pos += nn * sz
        trees.append(t)
    if pos != len(raw):
        raise ValueError("trailing bytes in model file")
    return trees


def write_model(path: str, trees) -> None:
    """Serialise a forest to the binary model format.  ``trees``: list of dicts with arrays feature (int32, -1 =
    leaf), threshold (float64), left, right, klass (int32)."""
    with open(path, "wb") as f:
        f.write(b"MOMDL1\0\0")
        f.write(np.array([1, 10, 6, len(trees)], dtype="<i4").tobytes())
        for t in trees:
            nn = len(t["feature"])
            f.write(np.array([nn], dtype="<i4").tobytes())
            f.write(np.asarray(t["feature"], dtype="<i4").tobytes())
            f.write(np.asarray(t["threshold"], dtype="<f8").tobytes())
            f.write(np.asarray(t["left"], dtype="<i4").tobytes())
            f.write(np.asarray(t["right"], dtype="<i4").tobytes())
            f.write(np.asarray(t["klass"], dtype="<i4").tobytes())


if torch.cuda.is_available():
    use_torch_allocator()
