"""GPU parity of the 4-bit floating-point (E2M1) flavour of the dense engine against the oracle.

The E2M1 value table used to decode bs_unpack_planes_fp4's output is the published format
(sign, two exponent bits with bias 1, one mantissa bit; subnormal 0.5): 0, 0.5, 1, 1.5, 2, 3, 4, 6."""
import numpy as np
import pytest
import torch

import oracle
import paper_1709_04060_amd as bs
from paper_1709_04060_amd import workloads
from gpu_util import FMT, assert_equal, dev, draw, planes_to_numpy, guarded_full

pytestmark = pytest.mark.gpu
U, TC, BP = oracle.UNSIGNED, oracle.TWOS_COMPLEMENT, oracle.BIPOLAR

E2M1 = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6, -0.0, -0.5, -1, -1.5, -2, -3, -4, -6], dtype=np.float64)
FP4_FORMATS = [(1, U), (1, TC), (1, BP), (2, U), (2, TC), (3, TC)]


def decode(codes: np.ndarray, depth: int) -> np.ndarray:
    """uint8 [rows][ld] of nibble pairs -> float values [rows][2 ld], low nibble first."""
    lo, hi = codes & 15, codes >> 4
    vals = np.stack([E2M1[lo], E2M1[hi]], axis=-1).reshape(codes.shape[0], -1)
    return vals


def to_fp4(X, bits, fmt):
    planes = bs.bs_pack_planes(dev(X.astype(np.int32)), bits, FMT[fmt])
    return bs.bs_unpack_planes_fp4(planes, FMT[fmt], X.shape[1])


@pytest.mark.parametrize("rows,depth", [(1, 1), (5, 31), (7, 32), (9, 33), (33, 130), (128, 1024), (300, 2400)])
@pytest.mark.parametrize("bits,fmt", FP4_FORMATS)
def test_unpack_fp4_decodes_to_the_packed_values(rows, depth, bits, fmt):
    rng = np.random.default_rng(rows + depth + bits)
    X = draw(rng, (rows, depth), bits, fmt)
    codes = to_fp4(X, bits, fmt).cpu().numpy()
    assert codes.shape[1] == 16 * ((depth + 31) // 32)
    vals = decode(codes, depth)
    assert_equal(vals[:, :depth].astype(np.int64), X.astype(np.int64), "unpack_fp4")
    nibbles = np.stack([codes & 15, codes >> 4], axis=-1).reshape(rows, -1)
    assert not nibbles[:, depth:].any()          # +0 (code 0), not -0, past the depth


@pytest.mark.parametrize("bits,fmt", [(3, U), (4, U), (4, TC)])
def test_unpack_fp4_refuses_values_outside_the_format(bits, fmt):
    X = draw(np.random.default_rng(0), (4, 64), bits, fmt)
    planes = bs.bs_pack_planes(dev(X.astype(np.int32)), bits, FMT[fmt])
    with pytest.raises(bs.BsError) as e:
        bs.bs_unpack_planes_fp4(planes, FMT[fmt], 64)
    assert e.value.status == bs.BS_ERR_UNSUPPORTED


@pytest.mark.parametrize("w,wf", FP4_FORMATS)
@pytest.mark.parametrize("a,af", FP4_FORMATS)
def test_gemm_fp4_all_formats(w, wf, a, af):
    rng = np.random.default_rng(w * 31 + a * 7 + wf + 3 * af)
    M, K, N = 70, 1100, 45                      # ragged everywhere, depth not a multiple of 128: register-staged kernel
    W, A = draw(rng, (M, K), w, wf), draw(rng, (K, N), a, af)
    C = bs.bs_gemm_fp4(to_fp4(W, w, wf), to_fp4(A.T.copy(), a, af), K)
    assert_equal(C.cpu().numpy(), oracle.gemm(W, A), "gemm_fp4 W%dA%d" % (w, a))


@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (32, 64, 32), (64, 128, 64), (100, 71, 45), (130, 1001, 257),
                                   (256, 256, 256), (300, 2400, 729), (1, 4096, 5), (513, 3, 9)])
def test_gemm_fp4_shapes(M, K, N):
    """Depths that are multiples of 128 take the direct-to-LDS kernel, the others the register-staged one; odd depths
    leave half a byte of padding in the last operand byte."""
    rng = np.random.default_rng(M + K + N)
    W, A = draw(rng, (M, K), 2, TC), draw(rng, (K, N), 2, U)
    C = bs.bs_gemm_fp4(to_fp4(W, 2, TC), to_fp4(A.T.copy(), 2, U), K)
    assert_equal(C.cpu().numpy(), oracle.gemm(W, A), "gemm_fp4 %dx%dx%d" % (M, K, N))


def test_gemm_fp4_extreme_values_deep():
    """Largest magnitudes of the supported formats at a depth where the sum needs 20 bits: -4 x 3 x 65536."""
    M, K, N = 40, 65536, 33
    W = np.full((M, K), -4, dtype=np.int8)
    A = np.full((K, N), 3, dtype=np.int8)
    C = bs.bs_gemm_fp4(to_fp4(W, 3, TC), to_fp4(A.T.copy(), 2, U), K).cpu().numpy()
    assert (C == -12 * K).all()
    A[:] = -4
    C = bs.bs_gemm_fp4(to_fp4(W, 3, TC), to_fp4(A.T.copy(), 3, TC), K).cpu().numpy()
    assert (C == 16 * K).all()


@pytest.mark.parametrize("M,K,N,obits", [(64, 256, 64, 2), (70, 1100, 45, 2), (200, 700, 130, 4), (260, 300, 3, 1),
                                         (513, 128, 300, 3)])
def test_gemm_fp4_threshold(M, K, N, obits):
    rng = np.random.default_rng(M + K + N + obits)
    W, A = draw(rng, (M, K), 1, BP), draw(rng, (K, N), 2, U)
    C = oracle.gemm(W, A)
    T = (1 << obits) - 1
    thr = np.sort(rng.integers(int(C.min()) - 2, int(C.max()) + 3, size=(M, T)), axis=1).astype(np.int32)
    out = guarded_full((obits, N, bs.bs_words_per_row(M)), -1, torch.int64)
    bs.bs_gemm_fp4_threshold(to_fp4(W, 1, BP), to_fp4(A.T.copy(), 2, U), K, dev(thr), obits, out=out)
    assert_equal(planes_to_numpy(out), oracle.threshold_pack(C, thr, obits), "gemm_fp4_threshold")


def test_fp4_engine_large_tiles_agree_with_the_other_engines():
    """2048^3 W2A2 takes the 256 x 256 tile configuration of the fp4 engine; all three engines give the same planes."""
    rng = np.random.default_rng(4096)
    n = 2048
    W, A = draw(rng, (n, n), 2, TC), draw(rng, (n, n), 2, U)
    Wp = bs.bs_pack_planes(dev(W), 2, bs.BS_TWOS_COMPLEMENT)
    Ap = bs.bs_pack_planes(dev(A), 2, bs.BS_UNSIGNED, depth_is_strided=True)
    W4, A4 = bs.bs_unpack_planes_fp4(Wp, bs.BS_TWOS_COMPLEMENT, n), bs.bs_unpack_planes_fp4(Ap, bs.BS_UNSIGNED, n)
    want = oracle.gemm(W, A)
    assert_equal(bs.bs_gemm_fp4(W4, A4, n).cpu().numpy(), want, "fp4 2048^3")
    thr = workloads.thresholds(rng, n, 2, float(want.mean()), float(want.std()))
    y4 = bs.bs_gemm_fp4_threshold(W4, A4, n, dev(thr), 2)
    y_bits = bs.bs_gemm_threshold(Wp, bs.BS_TWOS_COMPLEMENT, Ap, bs.BS_UNSIGNED, n, dev(thr), 2)
    assert_equal(planes_to_numpy(y4), oracle.threshold_pack(want, thr, 2), "fp4 fused")
    assert_equal(planes_to_numpy(y_bits), planes_to_numpy(y4), "engines agree")
