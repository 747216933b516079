"""Streamlining (Sec. 2.1): the library's host-side threshold computation against the float
pipeline evaluated directly in numpy (quantizer as thresholding, alpha-scaling, batch norm),
with the HWGQ quantizer of the paper's worked example.  No GPU needed."""
import numpy as np
import pytest

import oracle
import paper_1709_04060_amd as bs

HWGQ_T = np.array([0.0, 0.807, 1.345])       # thresholds of the 2-bit HWGQ quantizer (Sec. 2.1.1)
HWGQ_A, HWGQ_B = 0.538, 0.0                  # HWGQ(x) = 0.538 * T(x)


def float_layer(W, x_int, a_q, b_q, alpha, gamma, beta, mu, sigma, t):
    """The un-streamlined layer: float activations a_q x + b_q, matrix product, alpha-scaling,
    batch norm, then the quantizer's thresholding (values, not codes, are irrelevant here)."""
    z = W.astype(np.float64) @ (a_q * x_int.astype(np.float64) + b_q)
    z = alpha[:, None] * z
    y = gamma[:, None] * (z - mu[:, None]) / sigma[:, None] + beta[:, None]
    return y, oracle.threshold(y, np.tile(t, (W.shape[0], 1)))


@pytest.mark.parametrize("seed", range(5))
def test_streamlined_layer_equals_float_layer(seed):
    rng = np.random.default_rng(seed)
    M, K, N = 40, 300, 25
    W = (2 * rng.integers(0, 2, size=(M, K)) - 1).astype(np.int8)
    x = rng.integers(0, 4, size=(K, N)).astype(np.int8)
    alpha = rng.uniform(0.01, 0.2, size=M)
    gamma = rng.uniform(0.5, 2.0, size=M) * rng.choice([1.0, -1.0], size=M, p=[0.8, 0.2])   # some a < 0
    beta, mu, sigma = rng.normal(0.3, 0.5, size=M), rng.normal(0, 1.0, size=M), rng.uniform(0.5, 3.0, size=M)
    y, want = float_layer(W, x, HWGQ_A, HWGQ_B, alpha, gamma, beta, mu, sigma, HWGQ_T)
    a, b = bs.bs_streamline_collapse(M, HWGQ_A, HWGQ_B, W.sum(axis=1), alpha, gamma, beta, mu, sigma)
    acc = oracle.gemm(W, x)                                          # the integer accumulator
    assert np.allclose(a[:, None] * acc + b[:, None], y, rtol=1e-12, atol=1e-9)
    thr, neg = bs.bs_streamline_thresholds(HWGQ_T, a, b)
    assert np.array_equal(neg.astype(bool), a < 0)
    acc_eff = np.where(neg[:, None] == 1, -acc, acc)                  # negated channels: the caller negates the weight row
    got = oracle.threshold(acc_eff, thr)
    safe = np.abs(y[:, :, None] - HWGQ_T[None, None, :]).min(axis=2) > 1e-9   # away from float ties
    assert safe.mean() > 0.99
    assert np.array_equal(got[safe], want[safe])


def test_nonzero_quantizer_offset_uses_row_sums():
    rng = np.random.default_rng(9)
    M, K, N = 8, 64, 10
    W = rng.integers(-2, 2, size=(M, K)).astype(np.int8)
    x = rng.integers(0, 4, size=(K, N)).astype(np.int8)
    one, zero = np.ones(M), np.zeros(M)
    a_q, b_q = 0.25, -0.375                                           # dyadic: every product below is exact
    y, want = float_layer(W, x, a_q, b_q, one, one, zero, zero, one, np.array([-1.0, 0.5, 2.0]))
    a, b = bs.bs_streamline_collapse(M, a_q, b_q, W.sum(axis=1))
    assert np.array_equal(a, np.full(M, 0.25)) and np.array_equal(b, -0.375 * W.sum(axis=1))
    thr, neg = bs.bs_streamline_thresholds(np.array([-1.0, 0.5, 2.0]), a, b)
    assert not neg.any()
    assert np.array_equal(oracle.threshold(oracle.gemm(W, x), thr), want)   # exact arithmetic: ties included


def test_ceil_rule_and_special_cases():
    t = np.array([0.0, 0.807, 1.345])
    thr, neg = bs.bs_streamline_thresholds(t, np.array([0.538, 1.0, 2.0]), np.array([0.0, 0.0, 0.5]))
    assert thr.tolist() == [[0, 2, 3], [0, 1, 2], [0, 1, 1]]           # ceil(t / 0.538) = ceil(0, 1.5, 2.5); ceil((t - .5) / 2)
    assert not neg.any()
    thr, neg = bs.bs_streamline_thresholds(t, np.array([0.0, 0.0]), np.array([1.0, -1.0]))   # constant channels
    i32 = np.iinfo(np.int32)
    assert thr.tolist() == [[i32.min, i32.min, i32.max], [i32.max, i32.max, i32.max]]
    thr, neg = bs.bs_streamline_thresholds(t, np.array([-1.0]), np.array([0.0]))
    assert neg.tolist() == [1] and thr.tolist() == [[0, 1, 2]]        # -x >= ceil(t)
    thr, _ = bs.bs_streamline_thresholds(np.array([1e30, -1e30]), np.array([1.0]), np.array([0.0]))
    assert thr.tolist() == [[i32.max, i32.min]]                       # clamped


def test_argument_errors():
    lib = bs.load_library()
    assert lib.bs_streamline_thresholds(None, 3, None, None, 4, None, None) == bs.BS_ERR_INVALID_ARG
    t = np.array([0.0]); a = np.array([-1.0]); b = np.array([0.0]); thr = np.empty((1, 1), dtype=np.int32)
    p = lambda v: v.ctypes.data
    assert lib.bs_streamline_thresholds(p(t), 1, p(a), p(b), 1, p(thr), None) == bs.BS_ERR_UNSUPPORTED
