"""GPU parity of the dense (int8 MFMA) engine and of bs_unpack_planes against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_1709_04060_amd as bs
from paper_1709_04060_amd import workloads
from gpu_util import FMT, assert_equal, dev, draw, planes_to_numpy, guarded_full

pytestmark = pytest.mark.gpu
U, TC, BP = oracle.UNSIGNED, oracle.TWOS_COMPLEMENT, oracle.BIPOLAR


def padded(X, mult=16):
    """Rows padded to a multiple of `mult` with garbage the kernel must ignore."""
    r, k = X.shape
    ld = mult * ((k + mult - 1) // mult)
    out = np.full((r, ld), 77, dtype=np.int8)
    out[:, :k] = X
    return out


@pytest.mark.parametrize("rows,depth", [(1, 1), (5, 63), (7, 64), (33, 130), (128, 1024), (300, 2400)])
@pytest.mark.parametrize("bits,fmt", [(1, U), (2, U), (3, U), (4, U), (1, TC), (2, TC), (3, TC), (4, TC), (1, BP)])
def test_unpack_is_the_inverse_of_pack(rows, depth, bits, fmt):
    rng = np.random.default_rng(rows + depth + bits)
    X = draw(rng, (rows, depth), bits, fmt)
    planes = bs.bs_pack_planes(dev(X.astype(np.int32)), bits, FMT[fmt])
    got = bs.bs_unpack_planes(planes, FMT[fmt], depth).cpu().numpy()
    assert_equal(got[:, :depth], X, "unpack")
    assert not got[:, depth:].any()


@pytest.mark.parametrize("depth", [1, 15, 16, 17, 31, 33, 48, 100])
def test_unpack_leaves_the_row_padding_alone(depth):
    """A leading dimension wider than the depth: bytes up to the next multiple of 16 become 0, the rest stays."""
    import torch
    rng = np.random.default_rng(depth)
    X = draw(rng, (9, depth), 1, BP)
    planes = bs.bs_pack_planes(dev(X.astype(np.int32)), 1, FMT[BP])
    out = torch.full((9, 160), 77, dtype=torch.int8, device="cuda")
    got = bs.bs_unpack_planes(planes, FMT[BP], depth, out=out).cpu().numpy()
    edge = 16 * ((depth + 15) // 16)
    assert_equal(got[:, :depth], X, "unpack")
    assert not got[:, depth:edge].any()
    assert (got[:, edge:] == 77).all()


@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (32, 32, 32), (64, 64, 64), (100, 70, 45), (130, 1000, 257),
                                   (256, 128, 256), (300, 2400, 729), (1, 4096, 5)])
def test_gemm_i8_shapes(M, K, N):
    rng = np.random.default_rng(M + K + N)
    W = rng.integers(-8, 8, size=(M, K)).astype(np.int8)
    A = rng.integers(0, 16, size=(K, N)).astype(np.int8)
    Wd, Ad = dev(padded(W))[:, :], dev(padded(A.T.copy()))
    C = bs.bs_gemm_i8(Wd, Ad, K)
    assert_equal(C.cpu().numpy(), oracle.gemm(W, A), "gemm_i8 %dx%dx%d" % (M, K, N))


def test_gemm_i8_extreme_values():
    M, K, N = 70, 640, 50
    W = np.full((M, K), -128, dtype=np.int8)
    A = np.full((K, N), 127, dtype=np.int8)
    assert (bs.bs_gemm_i8(dev(W), dev(A.T.copy()), K).cpu().numpy() == -128 * 127 * K).all()
    W[:] = -128; A[:] = -128
    assert (bs.bs_gemm_i8(dev(W), dev(A.T.copy()), K).cpu().numpy() == 128 * 128 * K).all()


@pytest.mark.parametrize("M,K,N,obits", [(64, 256, 64, 2), (70, 1100, 45, 2), (200, 700, 130, 4), (260, 300, 3, 1),
                                         (513, 128, 300, 3)])
def test_gemm_i8_threshold(M, K, N, obits):
    rng = np.random.default_rng(M + K + N + obits)
    W = rng.integers(-8, 8, size=(M, K)).astype(np.int8)
    A = rng.integers(0, 16, size=(K, N)).astype(np.int8)
    C = oracle.gemm(W, A)
    T = (1 << obits) - 1
    thr = np.sort(rng.integers(int(C.min()) - 2, int(C.max()) + 3, size=(M, T)), axis=1).astype(np.int32)
    out = guarded_full((obits, N, bs.bs_words_per_row(M)), -1, torch.int64)
    bs.bs_gemm_i8_threshold(dev(padded(W)), dev(padded(A.T.copy())), K, dev(thr), obits, out=out)
    assert_equal(planes_to_numpy(out), oracle.threshold_pack(C, thr, obits), "gemm_i8_threshold")


def test_dense_engine_large_tiles_and_packed_route():
    """2048^3 (128 x 128 tiles, two workgroups per compute unit); operands come from packed planes through
    bs_unpack_planes, so the dense engine is checked as a drop-in for bs_gemm_threshold."""
    rng = np.random.default_rng(2048)
    n = 2048
    W = draw(rng, (n, n), 2, TC)
    A = draw(rng, (n, n), 2, U)
    Wp = bs.bs_pack_planes(dev(W), 2, bs.BS_TWOS_COMPLEMENT)
    Ap = bs.bs_pack_planes(dev(A), 2, bs.BS_UNSIGNED, depth_is_strided=True)
    W8 = bs.bs_unpack_planes(Wp, bs.BS_TWOS_COMPLEMENT, n)
    A8 = bs.bs_unpack_planes(Ap, bs.BS_UNSIGNED, n)            # [N][K]: the transposed activations
    C = bs.bs_gemm_i8(W8, A8, n)
    want = oracle.gemm(W, A)
    assert_equal(C.cpu().numpy(), want, "dense 2048^3")
    assert_equal(bs.bs_gemm(Wp, bs.BS_TWOS_COMPLEMENT, Ap, bs.BS_UNSIGNED, n).cpu().numpy(), want, "bit-serial 2048^3")
    thr = workloads.thresholds(rng, n, 2, float(want.mean()), float(want.std()))
    y_dense = bs.bs_gemm_i8_threshold(W8, A8, n, dev(thr), 2)
    y_bits = bs.bs_gemm_threshold(Wp, bs.BS_TWOS_COMPLEMENT, Ap, bs.BS_UNSIGNED, n, dev(thr), 2)
    assert_equal(planes_to_numpy(y_dense), oracle.threshold_pack(want, thr, 2), "dense fused")
    assert_equal(planes_to_numpy(y_bits), planes_to_numpy(y_dense), "engines agree")


@pytest.mark.parametrize("M,N", [(4096 - 3, 2304 - 5), (2048 - 3, 4096 - 5)])
def test_dense_engines_large_tiles(M, N):
    """The tile is chosen by rounds over the 256 compute units x relative round time (256 x 256: 1, 128 x 256: 0.6,
    128 x 128: 0.36).  4093 x 2299 outputs: 144 / 288 / 576 tiles -> 1 / 2 / 3 rounds -> the 256 x 256 tile;
    2045 x 4091: 128 / 256 / 512 tiles -> 1 / 1 / 2 rounds -> the 128 x 256 tile (smaller products take 128 x 128).
    int8 and fp4, int32 output and fused thresholds, ragged last tiles."""
    rng = np.random.default_rng(77 + M)
    K = 128
    W, A = draw(rng, (M, K), 2, TC), draw(rng, (K, N), 2, U)
    want = oracle.gemm(W, A)
    thr = workloads.thresholds(rng, M, 2, float(want.mean()), float(want.std()))
    wantp = oracle.threshold_pack(want, thr, 2)
    Wp = bs.bs_pack_planes(dev(W), 2, bs.BS_TWOS_COMPLEMENT)
    Ap = bs.bs_pack_planes(dev(A), 2, bs.BS_UNSIGNED, depth_is_strided=True)
    W8, A8 = bs.bs_unpack_planes(Wp, bs.BS_TWOS_COMPLEMENT, K), bs.bs_unpack_planes(Ap, bs.BS_UNSIGNED, K)
    assert_equal(bs.bs_gemm_i8(W8, A8, K).cpu().numpy(), want, "int8")
    assert_equal(planes_to_numpy(bs.bs_gemm_i8_threshold(W8, A8, K, dev(thr), 2)), wantp, "int8 fused")
    W4, A4 = bs.bs_unpack_planes_fp4(Wp, bs.BS_TWOS_COMPLEMENT, K), bs.bs_unpack_planes_fp4(Ap, bs.BS_UNSIGNED, K)
    assert_equal(bs.bs_gemm_fp4(W4, A4, K).cpu().numpy(), want, "fp4")
    assert_equal(planes_to_numpy(bs.bs_gemm_fp4_threshold(W4, A4, K, dev(thr), 2)), wantp, "fp4 fused")


@pytest.mark.parametrize("M,N", [(70, 45), (300, 520), (4096 - 3, 2304 - 5), (2048 - 3, 4096 - 5)])
@pytest.mark.parametrize("kbytes", [16, 48, 80, 144, 1200])
def test_dense_partial_last_stage(M, N, kbytes):
    """Depths of whole 16-byte chunks that are no multiple of the 64-byte stage (int8: K = kbytes, fp4: K = 2 kbytes;
    1200 bytes is conv2's lowered depth in E2M1 codes): the direct-to-LDS kernels complete the last stage with
    zeros.  Rows are followed in memory by a guard value that must not leak in; all three tile sizes."""
    rng = np.random.default_rng(M + N + kbytes)
    # int8 engine, operands with a leading dimension larger than the depth and guard bytes behind every row
    K = kbytes
    W, A = draw(rng, (M, K), 4, TC), draw(rng, (K, N), 4, U)
    want = oracle.gemm(W, A)
    Wg = np.full((M, K + 64), 99, dtype=np.int8); Wg[:, :K] = W
    Ag = np.full((N, K + 64), 99, dtype=np.int8); Ag[:, :K] = A.T
    Wd, Ad = dev(Wg)[:, :K], dev(Ag)[:, :K]                     # strided views: ld = K + 64
    assert_equal(bs.bs_gemm_i8(Wd, Ad, K).cpu().numpy(), want, "int8 %d bytes" % kbytes)
    thr = workloads.thresholds(rng, M, 4, float(want.mean()), float(want.std()) + 1.0)
    assert_equal(planes_to_numpy(bs.bs_gemm_i8_threshold(Wd, Ad, K, dev(thr), 4)), oracle.threshold_pack(want, thr, 4),
                 "int8 fused %d bytes" % kbytes)
    # fp4 engine from packed planes (the unpacker's rows are exactly K / 2 bytes)
    K = 2 * kbytes
    W, A = draw(rng, (M, K), 2, TC), draw(rng, (K, N), 2, U)
    want = oracle.gemm(W, A)
    W4 = bs.bs_unpack_planes_fp4(bs.bs_pack_planes(dev(W), 2, bs.BS_TWOS_COMPLEMENT), bs.BS_TWOS_COMPLEMENT, K)
    A4 = bs.bs_unpack_planes_fp4(bs.bs_pack_planes(dev(A), 2, bs.BS_UNSIGNED, depth_is_strided=True), bs.BS_UNSIGNED, K)
    assert_equal(bs.bs_gemm_fp4(W4, A4, K).cpu().numpy(), want, "fp4 %d bytes" % kbytes)
    thr = workloads.thresholds(rng, M, 2, float(want.mean()), float(want.std()) + 1.0)
    assert_equal(planes_to_numpy(bs.bs_gemm_fp4_threshold(W4, A4, K, dev(thr), 2)), oracle.threshold_pack(want, thr, 2),
                 "fp4 fused %d bytes" % kbytes)
