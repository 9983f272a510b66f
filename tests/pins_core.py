"""A compact run of the oracle's pins (dense brute force, closed forms, hand cases), callable against any build of
the oracle.  test_oracle_mutants.py runs it against deliberately broken copies of the oracle source to show that a
plausible mistake anywhere in it fails at least one pin."""
import math

import numpy as np

from oracle import ref
from paper_2303_05098_amd import synth
from tests import dense_pins

CASES = [(1, 9, 9, 0.3, 0.0), (2, 12, 7, 0.3, 0.3), (3, 5, 17, 0.5, 0.2), (4, 30, 30, 0.05, 0.0), (7, 24, 24, 0.6, 0.1)]


def check_all():
    # --- SpMV against dense matvec (rectangular cases catch transposition), |A||x| included
    for seed, m, n, dens, ef in CASES:
        m, n, rp, ci, v = synth.random_csr(m, n, dens, seed, ef)
        a, mask = dense_pins.dense_from_csr(m, n, rp, ci, v)
        x = synth.make_x(n, seed)
        ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
        perm = np.argsort(synth.uniform01(seed, 98, np.arange(ti.shape[0])))
        ti, tj, ta = ti[perm], tj[perm], ta[perm]
        y, mag = ref.spmv(m, n, ti, tj, ta, x)
        assert np.allclose(y, a @ x, rtol=0, atol=1e-14 * n)
        assert np.allclose(mag, np.abs(a) @ np.abs(x), rtol=1e-14, atol=0)
        # --- the multi-vector product against the dense product (k = 3, rectangular X catches a transposed layout)
        X = synth.uniform_pm1(seed, 41, np.arange(n * 3)).reshape(n, 3)
        Y, Mg = ref.spmm(m, n, ti, tj, ta, X)
        assert np.allclose(Y, a @ X, rtol=0, atol=1e-14 * n)
        assert np.allclose(Mg, np.abs(a) @ np.abs(X), rtol=1e-14, atol=0)
        # --- features, three thresholds
        for td in ((1, 2), (1, 4), (1, 1)):
            f, _ = ref.features(m, n, ti, tj, td)
            want = dense_pins.features(a, mask, td)
            for k in range(10):
                assert abs(f[k] - want[k]) <= 1e-14 * max(1.0, abs(want[k])), (k, f[k], want[k])
        # --- conversions by definition
        r, c, vv = ref.to_coo(ti, tj, ta)
        order = np.lexsort((tj, ti))
        assert np.array_equal(r, ti[order]) and np.array_equal(c, tj[order]) and np.array_equal(vv, ta[order])
        off, val = ref.to_dia(m, n, ti, tj, ta)
        woff, wval = dense_pins.dia(a, mask)
        assert np.array_equal(off, woff) and np.array_equal(val, wval)
        k, col, ev = ref.to_ell(m, ti, tj, ta)
        wk, wcol, wev, _ = dense_pins.ell(a, mask)
        assert k == wk and np.array_equal(col, wcol) and np.array_equal(ev, wev)
        for hyb in ((1, 3), (1, 2), (8, 9)):
            h = ref.to_hyb(m, ti, tj, ta, hyb)
            kk = dense_pins.hyb_k(mask, hyb)
            _, wcol, wev, rest = dense_pins.ell(a, mask, kk)
            assert h["k"] == kk and np.array_equal(h["ell_col"], wcol) and np.array_equal(h["ell_val"], wev)
            assert list(zip(h["coo_row"], h["coo_col"], h["coo_val"])) == [(i, j, x_) for i, j, x_ in rest]
        for td in ((1, 2), (1, 4), (1, 8)):
            d = ref.to_hdc(m, n, ti, tj, ta, td)
            woff, wval, wrp, wcol, wv = dense_pins.hdc(a, mask, td)
            assert np.array_equal(d["dia_off"], woff) and np.array_equal(d["dia_val"], wval)
            assert np.array_equal(d["csr_row_ptr"], wrp) and np.array_equal(d["csr_col"], wcol) and np.array_equal(d["csr_val"], wv)
    # --- back from every format: hand cases and round trips
    off = np.array([-1, 2], np.int32)
    dval = np.array([[9.0, 1.0, 2.0], [3.0, 0.0, 7.0]])
    got = sorted(zip(*[list(map(float, q)) for q in ref.from_dia(3, 4, off, dval)]))
    assert got == [(0.0, 2.0, 3.0), (1.0, 0.0, 1.0), (2.0, 1.0, 2.0)]
    ecol = np.array([[0, 2, -1], [3, -1, -1]], np.int32)
    ev = np.array([[5.0, 0.0, 0.0], [6.0, 0.0, 0.0]])
    got = sorted(zip(*[list(map(float, q)) for q in ref.from_ell(3, ecol, ev)]))
    assert got == [(0.0, 0.0, 5.0), (0.0, 3.0, 6.0), (1.0, 2.0, 0.0)]
    m, n, rp, ci, v = synth.random_csr(12, 7, 0.3, 2, 0.3)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    g = ref.from_csr(m, rp, ci, v)
    assert np.array_equal(g[0], ti) and np.array_equal(g[1], tj) and np.array_equal(g[2], ta)
    perm = np.argsort(synth.uniform01(5, 98, np.arange(ti.shape[0])))
    rp2, c2, v2 = ref.to_csr(m, ti[perm], tj[perm], ta[perm])
    assert np.array_equal(rp2, rp) and np.array_equal(c2, ci) and np.array_equal(v2, v)
    # --- closed forms: 5-point Laplacian 64 x 64
    m, n, rp, ci, v = synth.config(1)
    ti, tj, ta = ref.csr_to_triplets(rp, ci, v)
    f, ints = ref.features(m, n, ti, tj)
    assert list(f[:7]) == [4096, 4096, 20224, 4.9375, 20224 / 4096 ** 2, 5, 3]
    assert f[7] == math.sqrt(0.060546875) and f[8] == 5 and f[9] == 5 and ints["sum_sq_row"] == 100104
    y, _ = ref.spmv(m, n, ti, tj, ta, np.ones(n))
    assert y.sum() == 4 * 2 + 248 * 1
    # a band whose outer diagonals hold exactly half of min(M, N): still true diagonals (>=)
    mm, nn, rp, ci, v = synth.banded_scatter(8192, synth.C4_OFFSETS, 0, 100, 1)
    ti, tj, _ = ref.csr_to_triplets(rp, ci, v)
    assert ref.features(mm, nn, ti, tj)[0][9] == 9
    # --- K_H on a hand histogram
    lens = [5, 5, 5, 1, 1, 1, 1, 1, 0]
    t9 = np.repeat(np.arange(9, dtype=np.int32), lens)
    assert [ref.hyb_k(9, t9, h) for h in ((1, 3), (1, 2), (1, 1), (8, 9), (0, 1), (10, 9))] == [5, 1, 0, 1, 5, 0]
    # --- feasibility boundary
    assert ref.feasible(160, 10) and not ref.feasible(161, 10) and not ref.feasible(100, 10, 16, 99) and ref.feasible(99, 10, 16, 99)
    # --- tree walk, vote, ties
    leaf = lambda c: (-1, 0.0, -1, -1, c)  # noqa: E731

    def pack(trees):
        off, cols = [0], [[], [], [], [], []]
        for nodes in trees:
            for node in nodes:
                for q in range(5):
                    cols[q].append(node[q])
            off.append(len(cols[0]))
        return dict(tree_off=off, feature=cols[0], threshold=cols[1], left=cols[2], right=cols[3], klass=cols[4], n_classes=6)

    tree = [(3, 5.0, 1, 4, -1), (8, 2.0, 2, 3, -1), leaf(2), leaf(1), leaf(4)]
    x = np.zeros(10)
    x[3], x[8] = 5.0, 2.0
    assert ref.select(pack([tree]), x) == 2
    x[8] = 2.5
    assert ref.select(pack([tree]), x) == 1
    x[3] = 5.5
    assert ref.select(pack([tree]), x) == 4
    assert ref.select(pack([[leaf(5)], [leaf(1)]]), x) == 1
    assert ref.select(pack([[leaf(1)], [leaf(5)], [leaf(5)]]), x) == 5
    # --- run-first pick
    assert ref.pick([3.0, 2.0, 5.0, 2.0, 9.0, 4.0]) == 1
    assert ref.pick([np.nan, 2.0, 1.0, np.nan, 1.0, 4.0]) == 2
    assert ref.pick([np.nan] * 6) == -1
