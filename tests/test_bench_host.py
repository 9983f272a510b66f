"""Host-side checks of bench.py: the algorithmic bytes per SpMV (what each format has to move: x read once, y
written once, padding slots counted) against figures worked out by hand for the 27-point stencil on 128^3 and the
banded + scatter matrix, and the refusal of more than one GPU."""
import subprocess
import sys
from types import SimpleNamespace

import bench


def view(m, n, nnz, nd=0, k=0, nnz_coo=0, nnz_csr=0):
    return SimpleNamespace(m=m, n=n, nnz=nnz, nd=nd, k=k, nnz_coo=nnz_coo, nnz_csr=nnz_csr)


def test_algorithmic_bytes_of_the_stencil():
    m = n = 128 ** 3
    nnz = (3 * 128 - 2) ** 3                      # 27-point stencil: (3g - 2)^3 entries
    assert nnz == 55742968
    mb = lambda fmt, **kw: round(bench.algorithmic_bytes(fmt, view(m, n, nnz, **kw), 8) / 1e6, 1)  # noqa: E731
    assert mb(1, nnz_csr=nnz) == 710.9            # nnz * 12 + (m + 1) * 4 + 16 m
    assert mb(0, nnz_coo=nnz) == 925.4            # nnz * 16 + 16 m
    assert mb(2, nd=27) == 486.5                  # 27 m * 8 + 27 * 4 + 16 m
    assert mb(3, k=27) == 713.0                   # 27 m * 12 + 16 m
    assert mb(4, k=27) == 713.0                   # HYB that keeps every entry in its ELL part
    assert mb(5, nd=27) == 494.9                  # DIA part + the row pointer of an empty remainder


def test_algorithmic_bytes_of_the_banded_matrix():
    m = n = 4194304
    band = 9 * m - 2 * (1 + 2 + 2048 + 4096)
    scatter = band * 3 // 97
    nnz = band + scatter
    assert (scatter, nnz) == (1167106, 38903548)
    for sv, want_csr, want_hdc in ((8, 550.7, 399.9), (4, 361.6, 210.7)):
        assert round(bench.algorithmic_bytes(1, view(m, n, nnz, nnz_csr=nnz), sv) / 1e6, 1) == want_csr
        assert round(bench.algorithmic_bytes(5, view(m, n, nnz, nd=9, nnz_csr=scatter), sv) / 1e6, 1) == want_hdc


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, bench.__file__, "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr
