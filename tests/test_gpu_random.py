"""Seeded random sweep over shapes, precisions, formats and engines: every case compares the int32 product and the
fused thresholded planes of the GPU path with the oracle, element by element.  The draws put extra weight on the
sizes where the launch configuration changes (few columns, tile and word boundaries)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1709_04060_amd as bs
from gpu_util import FMT, assert_equal, conv_threshold_all_engines, dev, draw, gemm_all_engines, gemm_threshold_all_engines, guarded_full, planes_to_numpy

pytestmark = pytest.mark.gpu
U, TC, BP = oracle.UNSIGNED, oracle.TWOS_COMPLEMENT, oracle.BIPOLAR
EDGES = [1, 2, 3, 4, 5, 8, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257]


def draw_size(rng, hi):
    return int(rng.choice(EDGES)) if rng.random() < 0.5 else int(rng.integers(1, hi + 1))


def draw_operand(rng):
    fmt = [U, TC, BP][int(rng.integers(3))]
    bits = 1 if fmt == BP else int(rng.integers(1, 5))
    return bits, fmt


def make_case(seed):
    rng = np.random.default_rng([20240611, seed])
    (w, wf), (a, af) = draw_operand(rng), draw_operand(rng)
    M, N = draw_size(rng, 600), draw_size(rng, 600)
    K = int(rng.choice([1, 31, 32, 33, 64, 127, 128, 129, 1024, 1025])) if rng.random() < 0.4 else int(rng.integers(1, 4000))
    obits = int(rng.integers(1, 5))
    W, A = draw(rng, (M, K), w, wf), draw(rng, (K, N), a, af)
    C = oracle.gemm(W, A)
    T = (1 << obits) - 1
    thr = np.sort(rng.integers(int(C.min()) - 2, int(C.max()) + 3, size=(M, T)), axis=1).astype(np.int32)
    return rng, w, wf, a, af, M, K, N, obits, W, A, C, thr


@pytest.mark.parametrize("seed", range(120))
def test_random_bit_serial(seed):
    rng, w, wf, a, af, M, K, N, obits, W, A, C, thr = make_case(seed)
    what = "seed %d W%d(%d)A%d(%d) %dx%dx%d o=%d" % (seed, w, wf, a, af, M, K, N, obits)
    Wp = bs.bs_pack_planes(dev(W), w, FMT[wf])
    Ap = bs.bs_pack_planes(dev(A), a, FMT[af], depth_is_strided=True)
    assert_equal(gemm_all_engines(Wp, FMT[wf], Ap, FMT[af], K), C, "bs_gemm " + what)
    want = oracle.threshold_pack(C, thr, obits)
    assert_equal(gemm_threshold_all_engines(Wp, FMT[wf], Ap, FMT[af], K, dev(thr), obits), want, "bs_gemm_threshold " + what)
    out2 = guarded_full((obits, N, bs.bs_words_per_row(M)), -1, torch.int64)
    bs.bs_threshold_activate(dev(C), dev(thr), obits, out=out2)
    assert_equal(planes_to_numpy(out2), want, "bs_threshold_activate " + what)


@pytest.mark.parametrize("seed", range(120, 180))
def test_random_dense_engines(seed):
    """The int8 engine on every drawn case, the fp4 engine where both operands are E2M1-representable; both fed through
    the plane unpackers, so that the route bs_choose_engine may pick is the one under test."""
    rng, w, wf, a, af, M, K, N, obits, W, A, C, thr = make_case(seed)
    what = "seed %d W%d(%d)A%d(%d) %dx%dx%d o=%d" % (seed, w, wf, a, af, M, K, N, obits)
    Wp = bs.bs_pack_planes(dev(W), w, FMT[wf])
    Ap = bs.bs_pack_planes(dev(A.T.copy()), a, FMT[af])
    want = oracle.threshold_pack(C, thr, obits)
    W8, A8 = bs.bs_unpack_planes(Wp, FMT[wf], K), bs.bs_unpack_planes(Ap, FMT[af], K)
    assert_equal(bs.bs_gemm_i8(W8, A8, K).cpu().numpy(), C, "bs_gemm_i8 " + what)
    out = guarded_full((obits, N, bs.bs_words_per_row(M)), -1, torch.int64)
    bs.bs_gemm_i8_threshold(W8, A8, K, dev(thr), obits, out=out)
    assert_equal(planes_to_numpy(out), want, "bs_gemm_i8_threshold " + what)
    rep = lambda b, f: b <= 2 or (b == 3 and f == TC)
    if rep(w, wf) and rep(a, af):
        W4, A4 = bs.bs_unpack_planes_fp4(Wp, FMT[wf], K), bs.bs_unpack_planes_fp4(Ap, FMT[af], K)
        assert_equal(bs.bs_gemm_fp4(W4, A4, K).cpu().numpy(), C, "bs_gemm_fp4 " + what)
        out.fill_(-1)
        bs.bs_gemm_fp4_threshold(W4, A4, K, dev(thr), obits, out=out)
        assert_equal(planes_to_numpy(out), want, "bs_gemm_fp4_threshold " + what)


@pytest.mark.parametrize("seed", range(200, 240))
def test_random_convolution_and_pooling(seed):
    """Random geometries for the fused convolution (implicit lowering), the two-call route through the lowered matrix,
    and max pooling of the resulting packed map, against the direct convolution of the oracle."""
    rng = np.random.default_rng([20240611, seed])
    (w, wf), (a, af) = draw_operand(rng), draw_operand(rng)
    if af == BP:
        a, af = int(rng.integers(1, 5)), U         # image planes are unsigned or two's complement
    k = int(rng.choice([1, 2, 3, 5]))
    s, p = int(rng.integers(1, 4)), int(rng.integers(0, 3))
    H, W = int(rng.integers(k, 22)), int(rng.integers(k, 22))
    C = int(rng.choice([1, 3, 31, 32, 33, 64, 96, 130])) if rng.random() < 0.6 else int(rng.integers(1, 140))
    F = draw_size(rng, 300)
    obits = int(rng.integers(1, 5))
    x, filt = draw(rng, (H, W, C), a, af), draw(rng, (F, k, k, C), w, wf)
    conv = oracle.conv_direct(x, filt, s, p)
    OH, OW, _ = conv.shape
    Cmat = conv.reshape(OH * OW, F).T.copy()
    T = (1 << obits) - 1
    thr = np.sort(rng.integers(int(conv.min()) - 2, int(conv.max()) + 3, size=(F, T)), axis=1).astype(np.int32)
    want = oracle.threshold_pack(Cmat, thr, obits)
    what = "seed %d W%d(%d)A%d(%d) %dx%dx%d F=%d k=%d s=%d p=%d o=%d" % (seed, w, wf, a, af, H, W, C, F, k, s, p, obits)
    Cp = 32 * ((C + 31) // 32)
    fpad = np.zeros((F, k, k, Cp), dtype=filt.dtype)
    fpad[..., :C] = filt
    if wf == BP:
        fpad[..., C:] = -1                          # any value does: the activation pad bits are zero
    xp = bs.bs_pack_planes(dev(x.reshape(H * W, C)), a, FMT[af])
    Fp = bs.bs_pack_planes(dev(fpad.reshape(F, -1)), w, FMT[wf])
    got = conv_threshold_all_engines(xp, FMT[af], 1, H, W, C, Fp, FMT[wf], k, s, p, dev(thr), obits)
    assert_equal(got, want, "bs_conv_threshold " + what)
    low = bs.bs_im2col_interleaved(xp, H, W, C, k, k, s, p)
    two = bs.bs_gemm_threshold(Fp, FMT[wf], low, FMT[af], bs.bs_lowered_depth(C, k, k), dev(thr), obits)
    assert_equal(planes_to_numpy(two), want, "bs_im2col_interleaved + bs_gemm_threshold " + what)
    pk = int(rng.integers(1, 4))
    if pk <= min(OH, OW):
        ps = int(rng.integers(1, 3))
        Y = oracle.threshold(Cmat, thr).T.reshape(OH, OW, F)
        pooled = bs.bs_maxpool_packed(two, OH, OW, F, pk, ps)
        assert_equal(planes_to_numpy(pooled), oracle.pack(oracle.maxpool(Y, pk, ps).reshape(-1, F), obits, U), "bs_maxpool_packed " + what)


@pytest.mark.parametrize("seed", range(400, 460))
def test_random_pooled_convolution(seed):
    """Random batches, maps, pooling windows and kernels for the convolution that reads its input through a max pooling
    (including kernels that cover the whole pooled map, the fully connected case), against the oracle's pooling followed
    by its direct convolution."""
    rng = np.random.default_rng([20240611, seed])
    w, wf = draw_operand(rng)
    a, obits = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    B = int(rng.choice([1, 1, 2, 3, 4, 5, 9]))
    pk, ps = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    H, W = int(rng.integers(pk + 1, 20)), int(rng.integers(pk + 1, 20))
    PH, PW = (H - pk) // ps + 1, (W - pk) // ps + 1
    whole = rng.random() < 0.35 and PH == PW
    p = 0 if whole else int(rng.integers(0, 3))
    k = PH if whole else int(rng.choice([q for q in (1, 2, 3, 5) if q <= min(PH, PW) + 2 * p]))
    s = 1 if whole else int(rng.integers(1, 3))
    C = int(rng.choice([1, 3, 32, 33, 64, 96, 128, 130, 256])) if rng.random() < 0.7 else int(rng.integers(1, 140))
    F = draw_size(rng, 300)
    x, filt = draw(rng, (B, H, W, C), a, U), draw(rng, (F, k, k, C), w, wf)
    convs = [oracle.conv_direct(oracle.maxpool(x[b], pk, ps), filt, s, p) for b in range(B)]
    lo, hi = min(int(c.min()) for c in convs), max(int(c.max()) for c in convs)
    T = (1 << obits) - 1
    thr = np.sort(rng.integers(lo - 2, hi + 3, size=(F, T)), axis=1).astype(np.int32)
    OH, OW, _ = convs[0].shape
    want = np.concatenate([oracle.threshold_pack(c.reshape(OH * OW, F).T.copy(), thr, obits) for c in convs], axis=1)
    what = "seed %d W%d(%d)A%d B=%d %dx%dx%d pool %d/%d F=%d k=%d s=%d p=%d o=%d" % (seed, w, wf, a, B, H, W, C, pk, ps, F, k, s, p, obits)
    Cp = 32 * ((C + 31) // 32)
    fpad = np.zeros((F, k, k, Cp), dtype=filt.dtype)
    fpad[..., :C] = filt
    if wf == BP:
        fpad[..., C:] = -1
    xp = bs.bs_pack_planes(dev(x.reshape(B * H * W, C)), a, bs.BS_UNSIGNED)
    Fp = bs.bs_pack_planes(dev(fpad.reshape(F, -1)), w, FMT[wf])
    got = bs.bs_pool_conv_threshold_batch(xp, B, H, W, C, pk, ps, Fp, FMT[wf], k, k, s, p, dev(thr), obits)
    assert_equal(planes_to_numpy(got), want, "bs_pool_conv_threshold_batch " + what)


@pytest.mark.parametrize("seed", range(300, 364))
def test_random_large_shapes(seed):
    """Shapes beyond the sweep above, so that every tile configuration and both few-column kernels are drawn: mid-sized
    squares (32 x 16, 32 x 32 and 64 x 64 tiles), many rows with 1..40 columns, few rows with many columns.  Bit-serial
    and both matrix-core engines, int32 product and fused thresholds."""
    rng = np.random.default_rng([20240612, seed])
    (w, wf), (a, af) = draw_operand(rng), draw_operand(rng)
    regime = seed % 4
    if regime == 0:
        M, N = int(rng.integers(300, 1600)), int(rng.integers(300, 1600))
    elif regime == 1:
        M, N = int(rng.integers(1000, 20000)), int(rng.integers(1, 40))
    elif regime == 2:
        M, N = int(rng.integers(1, 400)), int(rng.integers(500, 8000))
    else:
        M, N = int(rng.integers(200, 1200)), int(rng.integers(200, 1200))
    K = int(rng.choice([32, 64, 96, 1024, 2048, 2400])) if rng.random() < 0.5 else int(rng.integers(1, 2500))
    K = max(1, min(K, int(2.5e9 / (M * N))))          # keeps the oracle's product to a few seconds
    obits = int(rng.integers(1, 5))
    W, A = draw(rng, (M, K), w, wf), draw(rng, (K, N), a, af)
    C = oracle.gemm(W, A)
    T = (1 << obits) - 1
    thr = np.sort(rng.integers(int(C.min()) - 2, int(C.max()) + 3, size=(M, T)), axis=1).astype(np.int32)
    want = oracle.threshold_pack(C, thr, obits)
    what = "seed %d W%d(%d)A%d(%d) %dx%dx%d o=%d" % (seed, w, wf, a, af, M, K, N, obits)
    Wp = bs.bs_pack_planes(dev(W), w, FMT[wf])
    Ap = bs.bs_pack_planes(dev(A), a, FMT[af], depth_is_strided=True)
    assert_equal(bs.bs_gemm(Wp, FMT[wf], Ap, FMT[af], K).cpu().numpy(), C, "bs_gemm " + what)
    out = guarded_full((obits, N, bs.bs_words_per_row(M)), -1, torch.int64)
    bs.bs_gemm_threshold(Wp, FMT[wf], Ap, FMT[af], K, dev(thr), obits, out=out)
    assert_equal(planes_to_numpy(out), want, "bs_gemm_threshold " + what)
    W8, A8 = bs.bs_unpack_planes(Wp, FMT[wf], K), bs.bs_unpack_planes(Ap, FMT[af], K)
    assert_equal(bs.bs_gemm_i8(W8, A8, K).cpu().numpy(), C, "bs_gemm_i8 " + what)
    out.fill_(-1)
    bs.bs_gemm_i8_threshold(W8, A8, K, dev(thr), obits, out=out)
    assert_equal(planes_to_numpy(out), want, "bs_gemm_i8_threshold " + what)
    rep = lambda b, f: b <= 2 or (b == 3 and f == TC)
    if rep(w, wf) and rep(a, af):
        W4, A4 = bs.bs_unpack_planes_fp4(Wp, FMT[wf], K), bs.bs_unpack_planes_fp4(Ap, FMT[af], K)
        assert_equal(bs.bs_gemm_fp4(W4, A4, K).cpu().numpy(), C, "bs_gemm_fp4 " + what)
        out.fill_(-1)
        bs.bs_gemm_fp4_threshold(W4, A4, K, dev(thr), obits, out=out)
        assert_equal(planes_to_numpy(out), want, "bs_gemm_fp4_threshold " + what)


@pytest.mark.parametrize("seed", range(500, 650))
def test_random_middle_shapes_on_every_engine(seed):
    """Up to 1700 rows and columns at any depth up to 3000: the matrix-core kernels' 64 x 64 and 128 x 128 tiles with
    up to several hundred workgroups, even and odd numbers of pipeline periods, every precision and format, the int32
    product and the fused thresholds on every engine."""
    rng = np.random.default_rng([20240613, seed])
    (w, wf), (a, af) = draw_operand(rng), draw_operand(rng)
    M, N = int(rng.integers(1, 1700)), int(rng.integers(5, 1700))
    K = int(rng.choice([64, 127, 128, 129, 255, 256, 257, 1024, 2304])) if rng.random() < 0.5 else int(rng.integers(1, 3000))
    obits = int(rng.integers(1, 5))
    W, A = draw(rng, (M, K), w, wf), draw(rng, (K, N), a, af)
    C = oracle.gemm(W, A)
    thr = np.sort(rng.integers(int(C.min()) - 2, int(C.max()) + 3, size=(M, (1 << obits) - 1)), axis=1).astype(np.int32)
    what = "seed %d W%d(%d)A%d(%d) %dx%dx%d o=%d" % (seed, w, wf, a, af, M, K, N, obits)
    Wp = bs.bs_pack_planes(dev(W), w, FMT[wf])
    Ap = bs.bs_pack_planes(dev(A), a, FMT[af], depth_is_strided=True)
    assert_equal(gemm_all_engines(Wp, FMT[wf], Ap, FMT[af], K), C, "bs_gemm " + what)
    assert_equal(gemm_threshold_all_engines(Wp, FMT[wf], Ap, FMT[af], K, dev(thr), obits), oracle.threshold_pack(C, thr, obits),
                 "bs_gemm_threshold " + what)
