"""The feature call that allocates nothing (mo_features_static) against mo_features and the oracle: two calls in a
row on the same GPU, the second on a smaller matrix, so that whatever the first call left in the library's device
array must not leak into the second; then an invalid matrix, and the size limit."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2303_05098_amd import mo, synth
from tests.gpu_util import upload

pytestmark = pytest.mark.gpu


def run_static(a, params=None):
    out = torch.full((mo.RESULT_BYTES,), 0xAB, dtype=torch.uint8, device="cuda")
    mo.mo_features_static(a, out, params)
    torch.cuda.synchronize()
    return mo.decode_feature_result(out.cpu().numpy().tobytes())


def check(m, n, rp, ci, v, params=None):
    a = upload(m, n, rp, ci, v)
    status, ints = run_static(a, params)
    assert status == mo.MO_OK
    f_lib, ints_lib = mo.mo_features(a, params)
    assert ints == ints_lib
    f = mo.mo_features_finalize(ints)
    assert f.tobytes() == f_lib.tobytes()
    ti, tj, _ = ref.csr_to_triplets(rp, ci, v)
    td = (params or {}).get("td_num", 1), (params or {}).get("td_den", 2)
    fo, io = ref.features(m, n, ti, tj, td)
    assert f.tobytes() == fo.tobytes() and ints == io


def test_two_calls_second_smaller():
    # first: lognormal rows, about 1.5 M entries spread over most of the 262 143 diagonals; second: a small Laplacian whose five diagonals lie inside the range just used
    m, n, rp, ci, v = synth.lognormal_rows(1 << 17, 11, mean=12.0, sigma=1.0)
    check(m, n, rp, ci, v)
    m, n, rp, ci, v = synth.config(1)
    check(m, n, rp, ci, v)
    # and a third, between the two in size, with another threshold for true diagonals
    m, n, rp, ci, v = synth.banded_scatter(50000, (0, 3, -3, 700, -1900), 5, 100, 5)
    check(m, n, rp, ci, v, {"td_num": 1, "td_den": 5})


def test_rows_too_long_for_one_wave():
    """Rows of 12 000 and 9 000 entries go through the list of deferred rows that lives in the same device array: twice, so
    that the second call finds the list as the first one left it, then with such a row out of order."""
    from tests.test_gpu_parity import bad_csr, very_long_rows
    m, n, rp, ci, v = very_long_rows()
    check(m, n, rp, ci, v)
    check(m, n, rp, ci, v)
    status, _ = run_static(upload(*bad_csr("vlong_unsorted")))
    assert status == mo.MO_E_CSR_INVALID
    check(m, n, rp, ci, v)


def test_largest_size_and_limit():
    m, n, rp, ci, v = synth.config(2)          # m + n - 1 = 4 194 303: just inside the limit
    assert m + n - 1 <= mo.STATIC_MAX_DIAGS
    check(m, n, rp, ci, v)
    # one past the limit: refused before anything is enqueued (the arrays need not even be that long)
    a = upload(m, n, rp, ci, v)
    a.n = mo.STATIC_MAX_DIAGS - m + 2
    out = torch.zeros(mo.RESULT_BYTES, dtype=torch.uint8, device="cuda")
    with pytest.raises(mo.MoError) as e:
        mo.mo_features_static(a, out)
    assert e.value.status == mo.MO_E_SHAPE
    assert not out.any()


def test_invalid_csr_is_reported_in_the_result():
    m, n, rp, ci, v = synth.config(1)
    ci = ci.copy()
    ci[7], ci[8] = ci[8], ci[7]                # columns out of order inside a row
    status, _ = run_static(upload(m, n, rp, ci, v))
    assert status == mo.MO_E_CSR_INVALID
    # the array is usable again right away
    m, n, rp, ci, v = synth.config(1)
    check(m, n, rp, ci, v)


def test_result_may_live_in_pinned_host_memory():
    m, n, rp, ci, v = synth.config(1)
    a = upload(m, n, rp, ci, v)
    host = torch.zeros(mo.RESULT_BYTES, dtype=torch.uint8).pin_memory()
    st = a.struct()
    rc = mo.lib.mo_features_static(C.byref(st), None, host.data_ptr(), int(torch.cuda.current_stream().cuda_stream))
    assert rc == mo.MO_OK
    torch.cuda.synchronize()
    status, ints = mo.decode_feature_result(host.numpy().tobytes())
    assert status == mo.MO_OK and ints == mo.mo_features(a)[1]
