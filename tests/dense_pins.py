"""Brute-force statements of every result on a dense matrix plus a stored-entry
mask.  Written straight from the format and feature definitions (Section II-B,
Table I) with numpy on dense arrays; used only to pin the CPU oracle on tiny
inputs.  Nothing here is shared with the oracle or with the GPU library."""
import numpy as np


def dense_from_csr(m, n, row_ptr, col_idx, val):
    a = np.zeros((m, n), dtype=np.float64)
    mask = np.zeros((m, n), dtype=bool)
    for i in range(m):
        for p in range(int(row_ptr[i]), int(row_ptr[i + 1])):
            a[i, int(col_idx[p])] = float(val[p])
            mask[i, int(col_idx[p])] = True
    return a, mask


def features(a, mask, td=(1, 2)):
    m, n = mask.shape
    lens = mask.sum(axis=1)
    nnz = int(mask.sum())
    avg = nnz / m
    cnts = [int(np.diagonal(mask, d).sum()) for d in range(-(m - 1), n)]
    n_d = sum(1 for c in cnts if c >= 1)
    n_td = sum(1 for c in cnts if c >= 1 and c * td[1] >= min(m, n) * td[0])
    std = float(np.sqrt(np.mean((lens - avg) ** 2)))
    return [m, n, nnz, avg, nnz / (m * n), int(lens.max()), int(lens.min()), std, n_d, n_td]


def dia(a, mask):
    m, n = mask.shape
    offs = [d for d in range(-(m - 1), n) if np.diagonal(mask, d).sum() >= 1]
    val = np.zeros((len(offs), m))
    for k, d in enumerate(offs):
        for i in range(m):
            j = i + d
            if 0 <= j < n and mask[i, j]:
                val[k, i] = a[i, j]
    return np.array(offs, dtype=np.int64), val


def ell(a, mask, k=None):
    m, n = mask.shape
    lens = mask.sum(axis=1)
    if k is None:
        k = int(lens.max()) if m else 0
    col = -np.ones((k, m), dtype=np.int64)
    val = np.zeros((k, m))
    rest = []
    for i in range(m):
        s = 0
        for j in range(n):
            if mask[i, j]:
                if s < k:
                    col[s, i] = j
                    val[s, i] = a[i, j]
                else:
                    rest.append((i, j, a[i, j]))
                s += 1
    return k, col, val, rest


def hyb_k(mask, hyb=(1, 3)):
    m = mask.shape[0]
    lens = mask.sum(axis=1)
    best = 0
    for k in range(0, int(lens.max()) + 1 if m else 1):
        if int((lens >= k).sum()) * hyb[1] >= m * hyb[0]:
            best = k
    return best


def hdc(a, mask, td=(1, 2)):
    m, n = mask.shape
    offs = []
    for d in range(-(m - 1), n):
        c = int(np.diagonal(mask, d).sum())
        if c >= 1 and c * td[1] >= min(m, n) * td[0]:
            offs.append(d)
    val = np.zeros((len(offs), m))
    rest_mask = mask.copy()
    for k, d in enumerate(offs):
        for i in range(m):
            j = i + d
            if 0 <= j < n and mask[i, j]:
                val[k, i] = a[i, j]
                rest_mask[i, j] = False
    row_ptr = np.zeros(m + 1, dtype=np.int64)
    col, v = [], []
    for i in range(m):
        for j in range(n):
            if rest_mask[i, j]:
                col.append(j)
                v.append(a[i, j])
        row_ptr[i + 1] = len(col)
    return np.array(offs, dtype=np.int64), val, row_ptr, np.array(col, dtype=np.int64), np.array(v)
