"""Mutation check of the oracle's pins (CPU only): every deliberately broken copy of the oracle source must fail the
pin run that the real oracle passes.  The mistakes are planted in the oracle, never in the GPU code."""
import ctypes as C
import os
import subprocess

import pytest

from oracle import ref
from tests import pins_core

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "mo_oracle.c")

MUTANTS = [
    ("spmv_transposed", "int64_t i = ti[t], j = tj[t];\n        if (i < 0 || i >= m || j < 0 || j >= n)", "int64_t i = tj[t], j = ti[t];\n        if (i < 0 || i >= m || j < 0 || j >= n)"),
    ("spmv_mag_signed", "mg[i] += fabsl(a) * fabsl(xv);", "mg[i] += a * xv;"),
    ("spmv_drops_first_term", "for (int64_t t = 0; t < nnz; ++t) {\n        int64_t i = ti[t], j = tj[t];", "for (int64_t t = 1; t < nnz; ++t) {\n        int64_t i = ti[t], j = tj[t];"),
    ("spmm_transposed_x", "long double xv = (long double)x[col * k + v];", "long double xv = (long double)x[v * n + col];"),
    ("spmm_transposed_a", "int64_t row = ti[e], col = tj[e];", "int64_t row = tj[e], col = ti[e];"),
    ("spmm_mag_signed", "abs_sum[row * k + v] += fabsl(a) * fabsl(xv);", "abs_sum[row * k + v] += a * xv;"),
    ("spmm_y_column_major", "sum[row * k + v] += a * xv;", "sum[v * m + row] += a * xv;"),
    ("avg_by_columns", "out[3] = (double)nnz / (double)m;", "out[3] = (double)nnz / (double)n;"),
    ("density_m_squared", "out[4] = (double)nnz / ((double)m * (double)n);", "out[4] = (double)nnz / ((double)m * (double)m);"),
    ("min_skips_empty_rows", "if (len[i] < mn) mn = len[i];", "if (len[i] < mn && len[i] > 0) mn = len[i];"),
    ("std_without_root", "out[7] = sqrt(var);", "out[7] = var;"),
    ("variance_without_mean", " - (unsigned __int128)nnz * (unsigned __int128)nnz;", ";"),
    ("variance_divisor_m_minus_1", "double var = (double)num / ((double)m * (double)m);", "double var = (double)num / ((double)m * (double)(m - 1));"),
    ("true_diag_strict", "return cnt >= 1 && (__int128)cnt * td_den >= (__int128)mn * td_num;", "return cnt >= 1 && (__int128)cnt * td_den > (__int128)mn * td_num;"),
    ("true_diag_uses_max_dim", "int64_t mn = m < n ? m : n;\n    return cnt >= 1", "int64_t mn = m > n ? m : n;\n    return cnt >= 1"),
    ("diag_offset_sign", "off[k] = (int32_t)(d - (m - 1));", "off[k] = (int32_t)((m - 1) - d);"),
    ("dia_fill_wrong_diagonal", "if (off[q] == d) { k = q; break; }", "if (off[q] == -d) { k = q; break; }"),
    ("dia_counts_only_nonneg", "int keep = all_nonempty ? (cnt[d] >= 1)", "int keep = all_nonempty ? (cnt[d] >= 2)"),
    ("ell_padding_zero_col", "col[s] = -1; val[s] = 0.0;", "col[s] = 0; val[s] = 0.0;"),
    ("ell_unsorted_rows", "if (a->j != b->j) return a->j < b->j ? -1 : 1;", "if (a->j != b->j) return a->j < b->j ? 1 : -1;"),
    ("coo_column_major", "if (a->i != b->i) return a->i < b->i ? -1 : 1;\n    if (a->j != b->j) return a->j < b->j ? -1 : 1;", "if (a->j != b->j) return a->j < b->j ? -1 : 1;\n    if (a->i != b->i) return a->i < b->i ? -1 : 1;"),
    ("hyb_k_strict", "if ((__int128)rows * hyb_den >= (__int128)m * hyb_num) best = k;", "if ((__int128)rows * hyb_den > (__int128)m * hyb_num) best = k;"),
    ("hyb_k_counts_longer_only", "if (len[i] >= k) rows++;", "if (len[i] > k) rows++;"),
    ("hdc_row_ptr_shifted", "for (int64_t t = 0; t < keep; ++t) row_ptr[s[t].i + 1]++;", "for (int64_t t = 0; t < keep; ++t) row_ptr[s[t].i]++;"),
    ("to_csr_row_ptr_shifted", "for (int64_t t = 0; t < nnz; ++t) row_ptr[s[t].i + 1]++;", "for (int64_t t = 0; t < nnz; ++t) row_ptr[s[t].i]++;"),
    ("from_dia_keeps_zeros", "if (val[k * m + i] == 0.0) continue;", ""),
    ("from_dia_keeps_columns_beyond_n", "if (j < 0 || j >= n) continue;", "if (j < 0) continue;"),
    ("from_dia_column_indexed", "if (ti) { ti[c] = (int32_t)i; tj[c] = (int32_t)j; ta[c] = val[k * m + i]; }", "if (ti) { ti[c] = (int32_t)j; tj[c] = (int32_t)i; ta[c] = val[k * m + i]; }"),
    ("from_ell_drops_column_zero", "if (col[s * m + i] < 0) continue;", "if (col[s * m + i] <= 0) continue;"),
    ("from_csr_skips_last_entry_of_row", "for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {", "for (int64_t p = row_ptr[i]; p + 1 < row_ptr[i + 1]; ++p) {"),
    ("feasible_non_strict", "if ((__int128)slots > (__int128)max_fill * nnz) return 0;", "if ((__int128)slots >= (__int128)max_fill * nnz) return 0;"),
    ("feasible_ignores_max_slots", "if (slots > max_slots) return 0;", ""),
    ("tree_strict_compare", "(x[f] <= threshold[base + node])", "(x[f] < threshold[base + node])"),
    ("tree_children_swapped", "? left[base + node] : right[base + node];", "? right[base + node] : left[base + node];"),
    ("vote_tie_to_highest", "if (votes[c] > votes[best]) best = c;", "if (votes[c] >= votes[best]) best = c;"),
    ("pick_tie_to_highest", "if (best < 0 || ms[k] < ms[best]) best = k;", "if (best < 0 || ms[k] <= ms[best]) best = k;"),
    ("pick_maximum", "if (best < 0 || ms[k] < ms[best]) best = k;", "if (best < 0 || ms[k] > ms[best]) best = k;"),
]


def load(path):
    lib = C.CDLL(path)
    lib.orc_dia_offsets.restype = C.c_int64
    lib.orc_max_row.restype = C.c_int64
    lib.orc_hyb_k.restype = C.c_int64
    for name in ("orc_from_dia", "orc_from_ell", "orc_from_csr"):
        getattr(lib, name).restype = C.c_int64
    return lib


def test_real_oracle_passes_the_pin_run():
    pins_core.check_all()


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, monkeypatch, name, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    c_path, so_path = str(tmp_path / "mut.c"), str(tmp_path / "libmut.so")
    open(c_path, "w").write(src.replace(old, new))
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-w", "-o", so_path, c_path, "-lm", "-lpthread"], check=True)
    ref.lib()                                  # make sure the real one is loaded before swapping
    monkeypatch.setattr(ref, "_lib", load(so_path))
    with pytest.raises((AssertionError, ValueError)):
        pins_core.check_all()
