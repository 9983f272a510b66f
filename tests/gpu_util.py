"""Shared helpers for the GPU parity tests: same seeded inputs to the HIP library and to the CPU oracle."""
import numpy as np
import torch

from oracle import ref
from paper_2303_05098_amd import mo

TOL = {np.float64: 1e-13, np.float32: 1e-5}     # max_i |y - y_ref|_i / (|A||x|)_i, as the benchmark spec fixes it


def upload(m, n, rp, ci, v, dtype=np.float64):
    return mo.Csr(m, n, rp, ci, np.asarray(v, dtype=dtype))


def oracle_inputs(rp, ci, v, x, dtype):
    """Triplets and x exactly as the GPU sees them (rounded to dtype, promoted back to fp64)."""
    ti, tj, ta = ref.csr_to_triplets(rp, ci, np.asarray(v, dtype=dtype).astype(np.float64))
    return ti, tj, ta, np.asarray(x, dtype=dtype).astype(np.float64)


def gpu_spmv(h, x_host, m, dtype):
    x = torch.as_tensor(np.asarray(x_host, dtype=dtype)).cuda()
    y = torch.full((m,), float("nan"), dtype=x.dtype, device="cuda")
    mo.mo_spmv(h, x, y)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def try_convert(a, fmt, params=None):
    try:
        return mo.mo_convert(a, fmt, params)
    except mo.MoError as e:
        if e.status == mo.MO_E_FILL:
            return None
        raise
