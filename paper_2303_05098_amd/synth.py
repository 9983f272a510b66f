"""Seeded synthetic CSR matrices shaped like the paper's SpMV workloads.

This module only *generates inputs*: it holds none of the method's arithmetic
(no SpMV, no conversion, no feature counting) and imports neither the HIP
binding nor the CPU oracle, so tests and the benchmark can feed the very same
arrays to both sides.  The paper profiles on ~2200 real square SuiteSparse
matrices (Section VII, "Setup"/"Format Distribution"); those are not available
offline, so the families below stand in for them: regular stencils (DIA/ELL
territory), power-law rows (HYB/CSR territory), banded-plus-scatter (HDC
territory) and uniform random rows.

Randomness is counter based: every number is a pure function of
(seed, stream, index), so any slice of a matrix can be regenerated on its own
and results do not depend on numpy's generator version.

Every generator returns ``(m, n, row_ptr, col_idx, val)`` with ``row_ptr`` and
``col_idx`` int32, ``val`` float64, columns strictly ascending inside a row.
"""
from __future__ import annotations

import math

import numpy as np

BASE_SEED = 230305098
X_SEED_OFFSET = 7

_U64 = np.uint64
_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _mix_int(z: int) -> int:
    z = (z + _GOLD) & _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def _mix_arr(z: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = z + _U64(_GOLD)
        z = (z ^ (z >> _U64(30))) * _U64(_C1)
        z = (z ^ (z >> _U64(27))) * _U64(_C2)
        return z ^ (z >> _U64(31))


def bits64(seed: int, stream: int, idx) -> np.ndarray:
    """64 pseudo-random bits for every entry of ``idx`` (any integer array)."""
    key = _mix_int(_mix_int(int(seed) & _M64) ^ (int(stream) & _M64))
    idx = np.asarray(idx).astype(np.uint64, copy=False)
    return _mix_arr(_mix_arr(idx ^ _U64(key)))


def uniform01(seed: int, stream: int, idx) -> np.ndarray:
    """Uniform doubles in [0, 1) with 53 random bits."""
    return (bits64(seed, stream, idx) >> _U64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def uniform_pm1(seed: int, stream: int, idx) -> np.ndarray:
    """Uniform doubles in [-1, 1)."""
    return 2.0 * uniform01(seed, stream, idx) - 1.0


def scalar01(seed: int, stream: int, idx: int) -> float:
    return float(uniform01(seed, stream, np.array([idx], dtype=np.uint64))[0])


def make_x(n: int, seed: int, dtype=np.float64) -> np.ndarray:
    """Input vector: uniform[-1,1) from ``seed + 7``."""
    x = uniform_pm1(seed + X_SEED_OFFSET, 0, np.arange(n, dtype=np.uint64))
    return x.astype(dtype)


def _csr_from_mask(cols2d: np.ndarray, mask2d: np.ndarray):
    """Rows are the first axis; keep masked entries in row-major order."""
    m = cols2d.shape[0]
    lens = mask2d.sum(axis=1, dtype=np.int64)
    row_ptr = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(lens, out=row_ptr[1:])
    col_idx = cols2d[mask2d].astype(np.int32)
    return row_ptr.astype(np.int32), col_idx


def laplace2d(nx: int, ny: int | None = None):
    """2-D 5-point Laplacian, row = iy*nx + ix, 4 on the diagonal, -1 on the
    four in-grid neighbours."""
    ny = nx if ny is None else ny
    m = nx * ny
    r = np.arange(m, dtype=np.int64)
    ix, iy = r % nx, r // nx
    offs = np.array([-nx, -1, 0, 1, nx], dtype=np.int64)
    cols = r[:, None] + offs[None, :]
    mask = np.stack([iy > 0, ix > 0, np.ones(m, bool), ix < nx - 1, iy < ny - 1], axis=1)
    row_ptr, col_idx = _csr_from_mask(cols, mask)
    vals2d = np.broadcast_to(np.array([-1.0, -1.0, 4.0, -1.0, -1.0]), cols.shape)
    val = np.ascontiguousarray(vals2d[mask], dtype=np.float64)
    return m, m, row_ptr, col_idx, val


def stencil27(g: int, seed: int):
    """3-D 27-point stencil on a g^3 grid, row = (iz*g + iy)*g + ix.  The 26
    off-centre values are uniform[-1,1); the centre is 1 + sum |off-centre
    values of that row| (strictly diagonally dominant)."""
    m = g * g * g
    r = np.arange(m, dtype=np.int64)
    ix, iy, iz = r % g, (r // g) % g, r // (g * g)
    d = np.array([-1, 0, 1], dtype=np.int64)
    dz, dy, dx = np.meshgrid(d, d, d, indexing="ij")
    dz, dy, dx = dz.ravel(), dy.ravel(), dx.ravel()          # ascending offset order
    offs = (dz * g + dy) * g + dx
    okx = [ix > 0, np.ones(m, bool), ix < g - 1]
    oky = [iy > 0, np.ones(m, bool), iy < g - 1]
    okz = [iz > 0, np.ones(m, bool), iz < g - 1]
    mask = np.empty((m, 27), dtype=bool)
    for k in range(27):
        mask[:, k] = okz[dz[k] + 1] & oky[dy[k] + 1] & okx[dx[k] + 1]
    cols = r[:, None] + offs[None, :]
    row_ptr, col_idx = _csr_from_mask(cols, mask)
    del cols
    slot = (r[:, None] * 27 + np.arange(27, dtype=np.int64)[None, :])
    v = uniform_pm1(seed, 1, slot.ravel()).reshape(m, 27)
    del slot
    v[:, 13] = 0.0
    v[~mask] = 0.0
    v[:, 13] = 1.0 + np.abs(v).sum(axis=1)
    val = np.ascontiguousarray(v[mask], dtype=np.float64)
    return m, m, row_ptr, col_idx, val


def _distinct_sorted_columns(lens: np.ndarray, n: int, seed: int, stream0: int):
    """For every row i draw lens[i] distinct uniform columns in [0,n), sorted."""
    m = lens.shape[0]
    row_ptr = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(lens, out=row_ptr[1:])
    nnz = int(row_ptr[-1])
    rows = np.repeat(np.arange(m, dtype=np.int64), lens)
    eid = np.arange(nnz, dtype=np.uint64)
    cols = np.minimum((uniform01(seed, stream0, eid) * n).astype(np.int64), n - 1)
    keys = rows * n + cols
    attempt = 0
    while True:
        keys.sort(kind="stable")
        dup = np.zeros(nnz, dtype=bool)
        if nnz > 1:
            dup[1:] = keys[1:] == keys[:-1]
        nd = int(dup.sum())
        if nd == 0:
            break
        attempt += 1
        where = np.nonzero(dup)[0]
        r = keys[where] // n
        c = np.minimum((uniform01(seed, stream0 + attempt, where.astype(np.uint64)) * n).astype(np.int64), n - 1)
        keys[where] = r * n + c
    col_idx = (keys - rows * n).astype(np.int32)
    return row_ptr.astype(np.int32), col_idx


def lognormal_rows(m: int, seed: int, mean: float = 16.0, sigma: float = 1.2, cap: int = 20000):
    """Power-law-like square matrix: row length = min(cap, round(exp(mu + sigma z)))
    with mu = ln(mean) - sigma^2/2 so that the distribution mean is ``mean``;
    columns distinct uniform, sorted; values uniform[-1,1).  Empty rows stay."""
    n = m
    idx = np.arange(m, dtype=np.uint64)
    u1 = np.maximum(uniform01(seed, 10, idx), 2.0 ** -53)
    u2 = uniform01(seed, 11, idx)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)
    mu = math.log(mean) - 0.5 * sigma * sigma
    lens = np.minimum(np.rint(np.exp(mu + sigma * z)), min(cap, n)).astype(np.int64)
    row_ptr, col_idx = _distinct_sorted_columns(lens, n, seed, 20)
    val = uniform_pm1(seed, 12, np.arange(col_idx.shape[0], dtype=np.uint64))
    return m, n, row_ptr, col_idx, val


def uniform_rows(m: int, k: int, seed: int):
    """Every row has exactly k distinct uniform columns."""
    k = min(k, m)
    lens = np.full(m, k, dtype=np.int64)
    row_ptr, col_idx = _distinct_sorted_columns(lens, m, seed, 20)
    val = uniform_pm1(seed, 12, np.arange(col_idx.shape[0], dtype=np.uint64))
    return m, m, row_ptr, col_idx, val


def banded_scatter(m: int, offsets, scatter_num: int, scatter_den: int, seed: int):
    """Square matrix with the given diagonals fully populated plus
    S = floor(band_nnz * scatter_num / (scatter_den - scatter_num)) entries at
    uniform random positions off the band (so scatter is scatter_num/scatter_den
    of the final nnz).  Values uniform[-1,1)."""
    n = m
    offsets = np.array(sorted(set(int(o) for o in offsets)), dtype=np.int64)
    offsets = offsets[np.abs(offsets) < m]
    r = np.arange(m, dtype=np.int64)
    band_keys = []
    for o in offsets:
        lo, hi = max(0, -int(o)), min(m, n - int(o))
        rr = r[lo:hi]
        band_keys.append(rr * n + rr + int(o))
    band_keys = np.concatenate(band_keys) if band_keys else np.zeros(0, np.int64)
    band_nnz = band_keys.shape[0]
    s_target = (band_nnz * scatter_num) // (scatter_den - scatter_num) if scatter_num > 0 else 0
    s_target = min(s_target, m * n - band_nnz)
    scat = np.zeros(0, dtype=np.int64)
    start = 0
    while scat.shape[0] < s_target:
        need = s_target - scat.shape[0]
        batch = int(need * 1.1) + 64
        cid = np.arange(start, start + batch, dtype=np.uint64)
        start += batch
        rr = np.minimum((uniform01(seed, 30, cid) * m).astype(np.int64), m - 1)
        cc = np.minimum((uniform01(seed, 31, cid) * n).astype(np.int64), n - 1)
        ok = ~np.isin(cc - rr, offsets)
        cand = (rr * n + cc)[ok]
        merged = np.concatenate([scat, cand])
        _, first = np.unique(merged, return_index=True)
        first.sort()
        scat = merged[first][:s_target]
    keys = np.concatenate([band_keys, scat])
    keys.sort()
    rows = keys // n
    col_idx = (keys - rows * n).astype(np.int32)
    lens = np.bincount(rows, minlength=m).astype(np.int64)
    row_ptr = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(lens, out=row_ptr[1:])
    val = uniform_pm1(seed, 12, np.arange(keys.shape[0], dtype=np.uint64))
    return m, n, row_ptr.astype(np.int32), col_idx, val


C4_OFFSETS = (0, 1, -1, 2, -2, 2048, -2048, 4096, -4096)


def config(c: int, scale: float = 1.0):
    """The four single-matrix benchmark configurations.  ``scale`` < 1 shrinks
    the matrix (same structure) for CPU-side tests."""
    seed = BASE_SEED + c
    if c == 1:
        g = max(4, int(round(64 * scale)))
        return laplace2d(g)
    if c == 2:
        g = max(3, int(round(128 * scale)))
        return stencil27(g, seed)
    if c == 3:
        m = max(64, int(round(1048576 * scale)))
        return lognormal_rows(m, seed)
    if c == 4:
        m = max(64, int(round(4194304 * scale)))
        return banded_scatter(m, C4_OFFSETS, 3, 100, seed)
    raise ValueError(f"unknown config {c}")


FAMILIES = ("laplace2d", "stencil27", "lognormal", "banded_scatter", "uniform_rows")


SWEEP_BASE = 2048          # matrices 0 .. 2047: the five families in rotation
SWEEP_EXTRA = 512          # matrices 2048 .. 2559: clustered bands and scaled copies of the four benchmark configurations


def _sweep_extra(k: int, n_lo: float, n_hi: float):
    """Matrices beyond the five rotating families.  Even k: a band whose diagonals come in clusters (a centre cluster
    and one to three pairs at +-d, every cluster 1, 3 or 5 diagonals wide, d a power of two times a small odd number),
    the shape of benchmark configuration 4, with 0 - 10 % scattered entries.  Odd k: benchmark configuration
    1 + (k >> 1) mod 4 at a size drawn log-uniformly (the first four odd k: at its own size)."""
    seed = BASE_SEED + 1000 + k
    n_t = math.exp(math.log(n_lo) + scalar01(seed, 40, 0) * (math.log(n_hi) - math.log(n_lo)))
    j = k - SWEEP_BASE
    if j % 2 == 1:
        c = 1 + (j >> 1) % 4
        native = {1: 4096.0, 2: 2097152.0, 3: 1048576.0, 4: 4194304.0}[c]
        if (j >> 1) < 4:
            scale = 1.0
        elif c == 1:
            scale = n_t ** 0.5 / 64.0
        elif c == 2:
            scale = n_t ** (1.0 / 3.0) / 128.0
        else:
            scale = min(n_t, native) / native
        return ("config%d_scaled" % c,) + config(c, scale)
    m = max(64, int(round(n_t)))
    pairs = 1 + int(scalar01(seed, 47, 0) * 3)                  # 1..3 pairs of off-centre clusters
    offs = []
    half = int(scalar01(seed, 48, 0) * 3)                        # centre cluster: 1, 3 or 5 wide
    offs += list(range(-half, half + 1))
    for q in range(pairs):
        d = (1 << (5 + int(scalar01(seed, 49, q) * 9))) * (1 + 2 * int(scalar01(seed, 50, q) * 2))   # 32 .. 8192, times 1 or 3
        w = int(scalar01(seed, 51, q) * 3)
        for o in range(-w, w + 1):
            offs += [d + o, -d + o]
    offs = [o for o in sorted(set(offs)) if abs(o) < m]
    pct = int(scalar01(seed, 45, 0) * 11)                        # 0..10 % scatter
    return ("banded_clustered",) + banded_scatter(m, offs, pct, 100, seed)


def sweep_matrix(k: int, n_lo: float = 1e3, n_hi: float = 4e6):
    """Matrix k of the tuner sweep: family = k mod 5, target n log-uniform in [n_lo, n_hi], except for the SWEEP_EXTRA
    indices from SWEEP_BASE on (see _sweep_extra).  Returns (family_name, m, n, row_ptr, col_idx, val)."""
    if SWEEP_BASE <= k < SWEEP_BASE + SWEEP_EXTRA:
        return _sweep_extra(k, n_lo, n_hi)
    seed = BASE_SEED + 1000 + k
    fam = FAMILIES[k % 5]
    n_t = math.exp(math.log(n_lo) + scalar01(seed, 40, 0) * (math.log(n_hi) - math.log(n_lo)))
    if fam == "laplace2d":
        return (fam,) + laplace2d(max(4, int(round(n_t ** 0.5))))
    if fam == "stencil27":
        return (fam,) + stencil27(max(3, int(round(n_t ** (1.0 / 3.0)))), seed)
    m = max(64, int(round(n_t)))
    if fam == "lognormal":
        mean = 4.0 + 28.0 * scalar01(seed, 41, 0)
        sigma = 0.5 + 1.0 * scalar01(seed, 42, 0)
        return (fam,) + lognormal_rows(m, seed, mean=mean, sigma=sigma)
    if fam == "banded_scatter":
        nd = 3 + int(scalar01(seed, 43, 0) * 13)          # 3..15 diagonals
        span = max(2, min(m - 1, 8192))
        raw = (uniform01(seed, 44, np.arange(4 * nd, dtype=np.uint64)) * (2 * span + 1)).astype(np.int64) - span
        offs = [0]
        for o in raw.tolist():
            if o not in offs:
                offs.append(o)
            if len(offs) == nd:
                break
        pct = int(scalar01(seed, 45, 0) * 11)              # 0..10 % scatter
        return (fam,) + banded_scatter(m, offs, pct, 100, seed)
    kk = 2 + int(scalar01(seed, 46, 0) * 63)               # 2..64 per row
    return (fam,) + uniform_rows(m, kk, seed)


def random_csr(m: int, n: int, density: float, seed: int, empty_row_frac: float = 0.0):
    """Small rectangular random CSR for property tests (Bernoulli pattern)."""
    idx = np.arange(m * n, dtype=np.uint64)
    mask = (uniform01(seed, 50, idx) < density).reshape(m, n)
    if empty_row_frac > 0:
        kill = uniform01(seed, 51, np.arange(m, dtype=np.uint64)) < empty_row_frac
        mask[kill, :] = False
    cols = np.broadcast_to(np.arange(n, dtype=np.int64)[None, :], (m, n))
    row_ptr, col_idx = _csr_from_mask(cols, mask)
    val = uniform_pm1(seed, 52, np.arange(col_idx.shape[0], dtype=np.uint64))
    return m, n, row_ptr, col_idx, val
