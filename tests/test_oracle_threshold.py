"""Pins for successive thresholding (O2, Sec. 2.1.1-2.1.3)."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hwgq_quantizer.txt")


def load_hwgq():
    scale, thr, rows = None, None, []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = line.split()
        if f[0] == "scale":
            scale = float(f[1])
        elif f[0] == "thresholds":
            thr = [float(v) for v in f[1:]]
        else:
            rows.append((float(f[0]), float(f[1]), float(f[2])))
    return scale, thr, rows


def test_hwgq_worked_example():
    """0.538 * T(x, {0, 0.807, 1.345}) reproduces the printed levels on each interval."""
    scale, thr, rows = load_hwgq()
    t = np.array([thr])
    for lo, hi, level in rows:
        lo_f = -5.0 if lo == -np.inf else lo
        hi_f = 5.0 if hi == np.inf else hi
        xs = np.linspace(lo_f, hi_f, 41)[1:-1]
        y = oracle.threshold(xs[None, :], t)
        assert np.allclose(scale * y, level), (lo, hi)


def test_count_equals_rank_and_monotone():
    rng = np.random.default_rng(0)
    for T in (1, 3, 7, 15):
        thr = np.sort(rng.integers(-30, 30, size=(9, T)), axis=1).astype(np.int32)
        C = np.tile(np.arange(-40, 41, dtype=np.int32), (9, 1))     # every value, exhaustive
        Y = oracle.threshold(C, thr)
        assert Y.min() >= 0 and Y.max() <= T
        assert (np.diff(Y.astype(np.int32), axis=1) >= 0).all()
        for m in range(9):
            assert np.array_equal(Y[m], np.searchsorted(thr[m], C[m], side="right"))
            assert np.array_equal(Y[m] == T, C[m] >= thr[m, -1])
            assert np.array_equal(Y[m] == 0, C[m] < thr[m, 0])


def test_thresholds_are_per_row_not_per_column():
    C = np.zeros((2, 3), dtype=np.int32)
    thr = np.array([[-1], [1]], dtype=np.int32)
    assert np.array_equal(oracle.threshold(C, thr), [[1, 1, 1], [0, 0, 0]])


def test_ceil_rounding_invariance_on_integers():
    """Integer inputs: rounding every threshold up changes nothing (Sec. 2.1.3)."""
    rng = np.random.default_rng(1)
    thr = np.sort(rng.normal(0, 20, size=(6, 3)), axis=1)
    C = rng.integers(-60, 60, size=(6, 500)).astype(np.int32)
    assert np.array_equal(oracle.threshold(C, thr), oracle.threshold(C, np.ceil(thr).astype(np.int32)))
    # rounding down is NOT invariant (the test would not notice a floor otherwise)
    thr2 = np.array([[0.5]])
    assert oracle.threshold(np.array([[0]]), thr2)[0, 0] != oracle.threshold(np.array([[0]]), np.floor(thr2))[0, 0]


def test_affine_absorption():
    """T(a x + b, t) = T(x, (t - b) / a) for a > 0 (Sec. 2.1.3)."""
    rng = np.random.default_rng(2)
    x = rng.integers(-100, 100, size=(4, 300)).astype(np.float64)
    t = np.sort(rng.normal(0, 1, size=(4, 3)), axis=1)
    for a, b in [(0.0371, -0.25), (2.0, 3.0), (0.538, 0.0)]:
        assert np.array_equal(oracle.threshold(a * x + b, t), oracle.threshold(x, (t - b) / a))


def test_threshold_pack_layout():
    """Plane p, column n, bit m = bit p of Y[m][n]; packed along the channel axis."""
    rng = np.random.default_rng(3)
    M, N = 70, 3
    C = rng.integers(-50, 50, size=(M, N)).astype(np.int32)
    thr = np.sort(rng.integers(-40, 40, size=(M, 3)), axis=1).astype(np.int32)
    Y = oracle.threshold(C, thr)
    P = oracle.threshold_pack(C, thr, 2)
    assert P.shape == (2, N, oracle.words_per_row(M))
    for p in range(2):
        for n in range(N):
            for m in range(M):
                bit = (int(P[p, n, m // 64]) >> (m % 64)) & 1
                assert bit == (int(Y[m, n]) >> p) & 1
