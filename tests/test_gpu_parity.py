"""GPU parity: every entry point of the C ABI against the CPU oracle, bit-exact,
element by element, on seeded inputs that span several tiles and ragged tails."""
import numpy as np
import pytest
import torch

import oracle
import paper_1709_04060_amd as bs
from gpu_util import (FMT, assert_equal, dev, draw, gemm_all_engines, gemm_threshold_all_engines, guarded_full, planes_to_dev,
                      planes_to_numpy)

pytestmark = pytest.mark.gpu
U, TC, BP = oracle.UNSIGNED, oracle.TWOS_COMPLEMENT, oracle.BIPOLAR


def make_thr(rng, C, obits):
    T = (1 << obits) - 1
    lo, hi = int(C.min()) - 2, int(C.max()) + 3
    return np.sort(rng.integers(lo, hi, size=(C.shape[0], T)), axis=1).astype(np.int32)


# ------------------------------------------------------------------ S1 pack
@pytest.mark.parametrize("rows,depth", [(1, 1), (3, 63), (5, 64), (7, 65), (64, 256), (130, 1000), (33, 4097)])
@pytest.mark.parametrize("bits,fmt", [(1, U), (2, U), (4, U), (2, TC), (3, TC), (4, TC), (1, BP)])
@pytest.mark.parametrize("dtype", [np.int8, np.int32])
def test_pack_rows_and_cols(rows, depth, bits, fmt, dtype):
    rng = np.random.default_rng(rows * 1000 + depth + bits)
    X = draw(rng, (rows, depth), bits, fmt).astype(dtype)
    want = oracle.pack(X, bits, fmt)
    got = bs.bs_pack_planes(dev(X), bits, FMT[fmt])
    assert_equal(planes_to_numpy(got), want, "pack depth-contiguous")
    got_t = bs.bs_pack_planes(dev(X.T.copy()), bits, FMT[fmt], depth_is_strided=True)
    assert_equal(planes_to_numpy(got_t), want, "pack depth-strided")


@pytest.mark.parametrize("rows,depth", [(4, 64), (132, 1008), (260, 2064), (128, 1024), (516, 80), (1024, 4096)])
@pytest.mark.parametrize("bits,fmt", [(1, U), (2, U), (4, U), (2, TC), (4, TC), (1, BP)])
@pytest.mark.parametrize("dtype", [np.int8, np.int32])
def test_pack_aligned_fast_paths(rows, depth, bits, fmt, dtype):
    """Shapes whose leading dimensions allow the vectorised kernels, with partial last
    words and partial row tiles; plus a sliced source whose last quad of rows is incomplete."""
    rng = np.random.default_rng(rows + depth + bits)
    X = draw(rng, (rows, depth), bits, fmt).astype(dtype)
    want = oracle.pack(X, bits, fmt)
    assert_equal(planes_to_numpy(bs.bs_pack_planes(dev(X), bits, FMT[fmt])), want, "fast pack rows")
    assert_equal(planes_to_numpy(bs.bs_pack_planes(dev(X.T.copy()), bits, FMT[fmt], depth_is_strided=True)), want,
                 "fast pack cols")
    sub = dev(X.T.copy())[:, : rows - 2]          # rows - 2 columns of a [depth][rows] buffer: ld stays aligned
    assert_equal(planes_to_numpy(bs.bs_pack_planes(sub, bits, FMT[fmt], depth_is_strided=True)),
                 oracle.pack(X[: rows - 2], bits, fmt), "fast pack cols, incomplete quad")


def test_pack_out_of_range_values_follow_the_documented_reduction():
    """Values outside the format's range keep their low bits; bipolar packs v > 0 as +1."""
    X = np.array([[-128, -3, -1, 0, 1, 2, 5, 127] * 8], dtype=np.int8)
    got = planes_to_numpy(bs.bs_pack_planes(dev(X), 1, bs.BS_BIPOLAR))
    want_bits = (X[0] > 0).astype(np.uint64)
    assert int(got[0, 0, 0]) == int(sum(int(b) << i for i, b in enumerate(want_bits)))
    got2 = planes_to_numpy(bs.bs_pack_planes(dev(X), 2, bs.BS_UNSIGNED))
    for p in range(2):
        assert int(got2[p, 0, 0]) == int(sum(((int(v) >> p) & 1) << i for i, v in enumerate(X[0].astype(np.int64) & 3)))
    got3 = planes_to_numpy(bs.bs_pack_planes(dev(X.T.copy()), 1, bs.BS_BIPOLAR, depth_is_strided=True))
    assert int(got3[0, 0, 0]) == int(got[0, 0, 0])


def test_pack_respects_leading_dimension_and_overwrites_padding():
    rng = np.random.default_rng(11)
    big = draw(rng, (40, 300), 2, U)
    X = big[:, :200]
    t = dev(big)[:, :200]                      # ld = 300 > depth
    out = guarded_full((2, 40, bs.bs_words_per_row(200)), -1, torch.int64)
    bs.bs_pack_planes(t, 2, bs.BS_UNSIGNED, out=out)
    assert_equal(planes_to_numpy(out), oracle.pack(X, 2, U), "pack with ld")
    tt = dev(big.T.copy())[:200, :]            # strided: [depth][rows], all 40 rows, ld = 40
    out.fill_(-1)
    bs.bs_pack_planes(tt, 2, bs.BS_UNSIGNED, depth_is_strided=True, out=out)
    assert_equal(planes_to_numpy(out), oracle.pack(X, 2, U), "pack strided with ld")


# ------------------------------------------------------------------ S3 + S4 GEMM
ALL_WA = [(w, wf, a, af) for w in (1, 2, 3, 4) for a in (1, 2, 3, 4) for wf in (U, TC) for af in (U, TC)]
BIP = [(1, BP, a, af) for a in (1, 2, 3, 4) for af in (U, TC)] + [(w, wf, 1, BP) for w in (1, 2, 3, 4) for wf in (U, TC)] \
      + [(1, BP, 1, BP)]


def run_gemm(W, A, w, wf, a, af):
    Wp = bs.bs_pack_planes(dev(W), w, FMT[wf])
    Ap = bs.bs_pack_planes(dev(A), a, FMT[af], depth_is_strided=True)
    # every engine that takes the case must give the same matrix (checked inside); the caller compares it with the oracle
    return gemm_all_engines(Wp, FMT[wf], Ap, FMT[af], W.shape[1])


@pytest.mark.parametrize("w,wf,a,af", ALL_WA + BIP)
def test_gemm_all_precisions_and_formats(w, wf, a, af):
    rng = np.random.default_rng(w * 64 + a * 16 + wf * 4 + af)
    M, K, N = 70, 1100, 45                      # ragged in every dimension, 2 depth stages
    W, A = draw(rng, (M, K), w, wf), draw(rng, (K, N), a, af)
    assert_equal(run_gemm(W, A, w, wf, a, af), oracle.gemm(W, A), "gemm W%dA%d" % (w, a))


@pytest.mark.parametrize("M,K,N", [(530, 1100, 610), (700, 1100, 900), (1500, 1100, 1480)])
@pytest.mark.parametrize("w,wf,a,af", ALL_WA + BIP)
def test_gemm_all_precisions_on_larger_grids(w, wf, a, af, M, K, N):
    """The launch configurations that small shapes do not reach: 340 tiles of 32 x 32 run as 32 x 16 tiles, 638 as
    32 x 32 tiles (both with the depth split over the wavefronts), and 576 tiles of 64 x 64; ragged in every dimension."""
    rng = np.random.default_rng(w * 64 + a * 16 + wf * 4 + af + M)
    W, A = draw(rng, (M, K), w, wf), draw(rng, (K, N), a, af)
    assert_equal(run_gemm(W, A, w, wf, a, af), oracle.gemm(W, A), "gemm W%dA%d %dx%dx%d" % (w, a, M, K, N))


@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (1, 64, 1), (64, 256, 64), (65, 129, 63), (200, 3000, 130),
                                   (257, 1024, 129), (31, 2049, 700), (1000, 100, 3), (3, 5000, 1000)])
@pytest.mark.parametrize("w,wf,a,af", [(1, BP, 2, U), (2, TC, 2, U), (4, TC, 4, U), (3, TC, 3, TC)])
def test_gemm_shapes(M, K, N, w, wf, a, af):
    rng = np.random.default_rng(M + K + N)
    W, A = draw(rng, (M, K), w, wf), draw(rng, (K, N), a, af)
    assert_equal(run_gemm(W, A, w, wf, a, af), oracle.gemm(W, A), "gemm %dx%dx%d" % (M, K, N))


@pytest.mark.parametrize("N", [1, 2, 3, 4, 5, 6, 7, 8, 9, 13, 16, 17])
@pytest.mark.parametrize("M,K", [(1, 1), (7, 64), (8, 130), (9, 1000), (100, 9216), (333, 4100)])
@pytest.mark.parametrize("w,wf,a,af,obits", [(1, BP, 2, U, 2), (4, TC, 4, U, 4), (2, U, 3, TC, 1), (3, TC, 1, U, 3),
                                             (1, U, 1, BP, 2)])
def test_few_column_path(N, M, K, w, wf, a, af, obits):
    """N <= 4 takes the streaming (GEMV) kernel, 5..16 columns too at these row counts (groups of four columns);
    N = 17 and bipolar activations the tiled one."""
    rng = np.random.default_rng(N * 100 + M + K + w)
    W, A = draw(rng, (M, K), w, wf), draw(rng, (K, N), a, af)
    want = oracle.gemm(W, A)
    assert_equal(run_gemm(W, A, w, wf, a, af), want, "gemv int32")
    thr = make_thr(rng, want, obits)
    Wp = bs.bs_pack_planes(dev(W), w, FMT[wf])
    Ap = bs.bs_pack_planes(dev(A), a, FMT[af], depth_is_strided=True)
    got = gemm_threshold_all_engines(Wp, FMT[wf], Ap, FMT[af], K, dev(thr), obits)
    assert_equal(got, oracle.threshold_pack(want, thr, obits), "gemv fused")


@pytest.mark.parametrize("N", [5, 8, 12, 16])
@pytest.mark.parametrize("w,wf,a,af,obits", [(1, BP, 2, U, 2), (4, TC, 4, U, 4)])
def test_few_columns_many_rows(N, w, wf, a, af, obits):
    """5..16 columns and many short rows: the time model hands these to the tiled kernel (32 x 8 tiles) instead of
    the grouped streaming kernel; 4096 x 256 for W4A4 and W1A2 lies on that side for every N here, 4096 x 9216 W4A4
    at N = 5 on the other."""
    rng = np.random.default_rng(N * 7 + w)
    for (M, K) in [(4096, 256), (4096 + 33, 9216 if (w == 4 and N == 5) else 300)]:
        W, A = draw(rng, (M, K), w, wf), draw(rng, (K, N), a, af)
        want = oracle.gemm(W, A)
        assert_equal(run_gemm(W, A, w, wf, a, af), want, "int32 %dx%dx%d" % (M, K, N))
        thr = make_thr(rng, want, obits)
        Wp = bs.bs_pack_planes(dev(W), w, FMT[wf])
        Ap = bs.bs_pack_planes(dev(A), a, FMT[af], depth_is_strided=True)
        got = gemm_threshold_all_engines(Wp, FMT[wf], Ap, FMT[af], K, dev(thr), obits)
        assert_equal(got, oracle.threshold_pack(want, thr, obits), "fused %dx%dx%d" % (M, K, N))


@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (64, 64, 64), (65, 129, 63), (200, 3000, 130), (4, 5000, 2), (300, 100, 4),
                                   (1024, 1024, 1024)])
def test_w1a1_bipolar_xor_path(M, K, N):
    """Both operands +-1: the XOR-popcount form, dot = K - 2 popcount(XOR) (tiled and few-column kernels)."""
    rng = np.random.default_rng(M * 3 + K + N)
    W, A = draw(rng, (M, K), 1, BP), draw(rng, (K, N), 1, BP)
    want = oracle.gemm(W, A)
    assert_equal(run_gemm(W, A, 1, BP, 1, BP), want, "W1A1 int32")
    thr = make_thr(rng, want, 1)
    Wp = bs.bs_pack_planes(dev(W), 1, bs.BS_BIPOLAR)
    Ap = bs.bs_pack_planes(dev(A), 1, bs.BS_BIPOLAR, depth_is_strided=True)
    assert_equal(gemm_threshold_all_engines(Wp, bs.BS_BIPOLAR, Ap, bs.BS_BIPOLAR, K, dev(thr), 1),
                 oracle.threshold_pack(want, thr, 1), "W1A1 fused")
    got = bs.bs_gemm_threshold(Wp, bs.BS_BIPOLAR, Ap, bs.BS_BIPOLAR, K, dev(thr), 1)
    # a binarised layer chains: the 1-bit output planes are the next layer's bipolar operand
    W2 = draw(rng, (33, M), 1, BP)
    want2 = oracle.gemm(W2, (2 * oracle.threshold(want, thr).astype(np.int8) - 1))
    got2 = gemm_all_engines(bs.bs_pack_planes(dev(W2), 1, bs.BS_BIPOLAR), bs.BS_BIPOLAR, got, bs.BS_BIPOLAR, M)
    assert_equal(got2, want2, "W1A1 chained")


@pytest.mark.parametrize("w,wf,a,af", [(2, TC, 2, U), (4, TC, 4, U), (3, U, 4, TC), (4, U, 1, U)])
@pytest.mark.parametrize("M,K,N", [(70, 1100, 45), (130, 2000, 3), (64, 4096, 600)])
def test_gemm_topbits(w, wf, a, af, M, K, N):
    rng = np.random.default_rng(w + a + M + N)
    W, A = draw(rng, (M, K), w, wf), draw(rng, (K, N), a, af)
    Wp = bs.bs_pack_planes(dev(W), w, FMT[wf])
    Ap = bs.bs_pack_planes(dev(A), a, FMT[af], depth_is_strided=True)
    Wo, Ao = oracle.pack(W, w, wf), oracle.pack(A.T, a, af)
    for s in range(0, w + a - 1):
        got = bs.bs_gemm_topbits(Wp, FMT[wf], Ap, FMT[af], K, s).cpu().numpy()
        want = oracle.bitserial_gemm_topbits(Wo, wf == TC, Ao, af == TC, s)
        assert_equal(got.astype(np.int64), want, "topbits min_shift=%d" % s)


@pytest.mark.parametrize("N", [1, 6])
@pytest.mark.parametrize("K", [1 << 22, 17895697])
def test_gemm_very_deep_extreme_values(N, K):
    """Extremal W4A4 values through thousands of depth stages (few-column kernel for N = 1, tiled kernel for N = 6,
    the int8 matrix-core kernel for both).  K = 17895697 is the deepest product the library accepts for these
    formats: |C| = 8 * 15 * K = 2147483640 <= 2^31 - 1, so partial sums of plane-pair terms wrap around on the way
    and the result must still be exact."""
    M = 5
    rng = np.random.default_rng(N)
    W = np.full((M, K), -8, dtype=np.int8)
    A = np.full((K, N), 15, dtype=np.int8)
    W[1] = draw(rng, (K,), 4, TC)
    W[2] = 7
    if N > 1:
        A[:, -1] = draw(rng, (K,), 4, U)
    Wp = bs.bs_pack_planes(dev(W), 4, bs.BS_TWOS_COMPLEMENT)
    # packed from the transposed copy: the transposing pack walks the depth in the launch grid's second dimension,
    # which this depth exceeds for a source without 4-element alignment (it is refused there)
    Ap = bs.bs_pack_planes(dev(np.ascontiguousarray(A.T)), 4, bs.BS_UNSIGNED)
    got = gemm_all_engines(Wp, bs.BS_TWOS_COMPLEMENT, Ap, bs.BS_UNSIGNED, K)
    assert_equal(got, oracle.gemm(W, A), "deep W4A4")
    assert got[0, 0] == -8 * 15 * K and got[2, 0] == 7 * 15 * K
    # 2^31 / (8 * 15) = 17895697.07: one index more is refused (the argument check alone is exercised here)
    lib = bs.load_library()
    assert lib.bs_gemm(Wp.data_ptr(), 4, 1, Ap.data_ptr(), 4, 0, M, N, 17895698, got.ctypes.data, N, None) \
        == bs.BS_ERR_OVERFLOW_RISK


def test_gemm_extreme_values_and_ldc():
    M, K, N = 66, 640, 50
    for w, a in [(2, 2), (4, 4)]:
        W = np.full((M, K), -(1 << (w - 1)), dtype=np.int8)
        A = np.full((K, N), (1 << a) - 1, dtype=np.int8)
        assert (run_gemm(W, A, w, TC, a, U) == -K * (1 << (w - 1)) * ((1 << a) - 1)).all()
    rng = np.random.default_rng(5)
    W, A = draw(rng, (M, K), 2, TC), draw(rng, (K, N), 2, U)
    Wp = bs.bs_pack_planes(dev(W), 2, bs.BS_TWOS_COMPLEMENT)
    Ap = bs.bs_pack_planes(dev(A), 2, bs.BS_UNSIGNED, depth_is_strided=True)
    big = torch.full((M, 77), 123456, dtype=torch.int32, device="cuda")
    bs.bs_gemm(Wp, bs.BS_TWOS_COMPLEMENT, Ap, bs.BS_UNSIGNED, K, out=big[:, :N])     # ldc = 77, unaligned rows
    got = big.cpu().numpy()
    assert_equal(got[:, :N], oracle.gemm(W, A), "gemm ldc")
    assert (got[:, N:] == 123456).all()         # nothing written beyond N


# ------------------------------------------------------------------ S5 threshold
@pytest.mark.parametrize("M,N", [(1, 1), (64, 64), (70, 45), (129, 300), (300, 2), (4096, 1)])
@pytest.mark.parametrize("obits", [1, 2, 3, 4])
def test_threshold_activate(M, N, obits):
    rng = np.random.default_rng(M * 7 + N + obits)
    C = rng.integers(-500, 500, size=(M, N)).astype(np.int32)
    thr = make_thr(rng, C, obits)
    out = guarded_full((obits, N, bs.bs_words_per_row(M)), -1, torch.int64)
    bs.bs_threshold_activate(dev(C), dev(thr), obits, out=out)
    assert_equal(planes_to_numpy(out), oracle.threshold_pack(C, thr, obits), "threshold")


# tiny grids take 32 x 8 tiles, (530, 1100, 610) 32 x 16, (700, 600, 900) 32 x 32, (1500, 700, 1480) 64 x 64 ones
@pytest.mark.parametrize("M,K,N", [(1, 64, 1), (64, 256, 64), (70, 1100, 45), (200, 700, 130), (260, 300, 3), (530, 1100, 610),
                                   (700, 600, 900), (1500, 700, 1480)])
@pytest.mark.parametrize("w,wf,a,af,obits", [(1, BP, 2, U, 2), (2, TC, 2, U, 2), (4, TC, 4, U, 4), (1, BP, 1, BP, 1),
                                             (2, U, 3, TC, 3)])
def test_gemm_threshold_fused(M, K, N, w, wf, a, af, obits):
    rng = np.random.default_rng(M + K + N + obits)
    W, A = draw(rng, (M, K), w, wf), draw(rng, (K, N), a, af)
    C = oracle.gemm(W, A)
    thr = make_thr(rng, C, obits)
    Wp = bs.bs_pack_planes(dev(W), w, FMT[wf])
    Ap = bs.bs_pack_planes(dev(A), a, FMT[af], depth_is_strided=True)
    got = gemm_threshold_all_engines(Wp, FMT[wf], Ap, FMT[af], K, dev(thr), obits)
    assert_equal(got, oracle.threshold_pack(C, thr, obits), "fused gemm+threshold")


def test_fused_int8_planes_676_small_tiles_odd_period_count():
    """W3A3 1620 x 2831 x 1657 with 4-bit outputs: 676 tiles of 64 x 64 on the int8 matrix-core kernel, an odd number of
    periods, so that the loader's last two-period request is never read back; the per-row terms of the epilogue take
    the place of the stashed plane words and must not be written before that request has landed (a run once produced
    all-ones words in 96 columns of one tile row)."""
    rng = np.random.default_rng(420)
    M, K, N, obits = 1620, 2831, 1657, 4
    W, A = draw(rng, (M, K), 3, TC), draw(rng, (K, N), 3, U)
    C = oracle.gemm(W, A)
    thr = make_thr(rng, C, obits)
    Wp = bs.bs_pack_planes(dev(W), 3, FMT[TC])
    Ap = bs.bs_pack_planes(dev(A), 3, FMT[U], depth_is_strided=True)
    want = oracle.threshold_pack(C, thr, obits)
    for _ in range(3):
        assert_equal(gemm_threshold_all_engines(Wp, FMT[TC], Ap, FMT[U], K, dev(thr), obits), want, "fused W3A3 1620x2831x1657")


@pytest.mark.parametrize("K", [1, 64, 129, 257, 385, 513, 641])
@pytest.mark.parametrize("w,wf,a,af,obits", [(2, TC, 2, U, 2), (4, TC, 4, U, 4), (1, BP, 1, BP, 1)])
def test_large_tiles_short_depths(K, w, wf, a, af, obits):
    """2500 x 5000 outputs take the matrix-core kernels' 256 x 256 tiles, whose two groups of wavefronts run the period
    with different schedules (one expands a stage ahead of the other): one to five stages, whole and partial, so that
    prologue, tail and the stages past the depth of either schedule are what is exercised."""
    rng = np.random.default_rng(7000 + K + w)
    M, N = 2500, 5000
    W, A = draw(rng, (M, K), w, wf), draw(rng, (K, N), a, af)
    C = oracle.gemm(W, A)
    thr = make_thr(rng, C, obits)
    Wp = bs.bs_pack_planes(dev(W), w, FMT[wf])
    Ap = bs.bs_pack_planes(dev(A), a, FMT[af], depth_is_strided=True)
    assert_equal(gemm_all_engines(Wp, FMT[wf], Ap, FMT[af], K), C, "gemm 2500x%dx5000" % K)
    assert_equal(gemm_threshold_all_engines(Wp, FMT[wf], Ap, FMT[af], K, dev(thr), obits), oracle.threshold_pack(C, thr, obits),
                 "fused gemm+threshold 2500x%dx5000" % K)


# Long, thin outputs: the matrix-core kernels on packed planes map their workgroups to tiles in one of three orders
# (plain; runs of consecutive tiles per XCD, by rows or by columns of the tile grid), chosen on the host from the grid
# and the operands' planes.  These shapes reach the two run orders with every tile size, ragged edges, a tile count
# that is no multiple of 8 and more tiles than the chip holds at a time.
@pytest.mark.parametrize("M,K,N", [(390, 200, 10801), (70, 130, 16390), (16390, 130, 70), (200, 96, 43270), (43270, 96, 200),
                                   (384, 192, 43264), (8200, 300, 390), (1030, 260, 4100), (600, 64, 43270), (43270, 64, 600)])
@pytest.mark.parametrize("w,wf,a,af,obits", [(1, BP, 2, U, 2), (2, TC, 2, U, 2), (4, TC, 4, U, 4)])
def test_long_thin_outputs_on_every_engine(M, K, N, w, wf, a, af, obits):
    rng = np.random.default_rng(M + 3 * K + 7 * N + obits)
    W, A = draw(rng, (M, K), w, wf), draw(rng, (K, N), a, af)
    C = oracle.gemm(W, A)
    thr = make_thr(rng, C, obits)
    Wp = bs.bs_pack_planes(dev(W), w, FMT[wf])
    Ap = bs.bs_pack_planes(dev(A), a, FMT[af], depth_is_strided=True)
    assert_equal(gemm_all_engines(Wp, FMT[wf], Ap, FMT[af], K), C, "long thin gemm %dx%dx%d" % (M, K, N))
    got = gemm_threshold_all_engines(Wp, FMT[wf], Ap, FMT[af], K, dev(thr), obits)
    want = oracle.threshold_pack(C, thr, obits)
    assert_equal(got, want, "long thin fused gemm+threshold %dx%dx%d" % (M, K, N))
    # the kernels on unpacked operands order their tiles the same way
    W8, A8 = bs.bs_unpack_planes(Wp, FMT[wf], K), bs.bs_unpack_planes(Ap, FMT[af], K)
    assert_equal(bs.bs_gemm_i8(W8, A8, K).cpu().numpy(), C, "long thin bs_gemm_i8 %dx%dx%d" % (M, K, N))
    assert_equal(planes_to_numpy(bs.bs_gemm_i8_threshold(W8, A8, K, dev(thr), obits)), want, "long thin bs_gemm_i8_threshold")
    if w <= 2 and a <= 2:
        W4, A4 = bs.bs_unpack_planes_fp4(Wp, FMT[wf], K), bs.bs_unpack_planes_fp4(Ap, FMT[af], K)
        assert_equal(planes_to_numpy(bs.bs_gemm_fp4_threshold(W4, A4, K, dev(thr), obits)), want, "long thin bs_gemm_fp4_threshold")


# ------------------------------------------------------------------ S2 lowering
def pad_channels(x, Cp):
    out = np.zeros(x.shape[:-1] + (Cp,), dtype=x.dtype)
    out[..., : x.shape[-1]] = x
    return out


@pytest.mark.parametrize("H,W,C,k,s,p", [(5, 6, 3, 3, 1, 1), (7, 7, 32, 5, 1, 2), (9, 8, 40, 3, 2, 0),
                                         (6, 6, 96, 1, 1, 0), (27, 27, 96, 5, 1, 2), (8, 9, 130, 3, 2, 1)])
@pytest.mark.parametrize("abits", [1, 2, 4])
def test_im2col_interleaved(H, W, C, k, s, p, abits):
    rng = np.random.default_rng(H * W + C + abits)
    x = draw(rng, (H, W, C), abits, U)
    Cp = 32 * ((C + 31) // 32)
    # expected: plain lowering of the channel-padded image, then packed column by column
    L = oracle.im2col_plain(pad_channels(x, Cp), k, k, s, p)
    assert L.shape[0] == bs.bs_lowered_depth(C, k, k)
    want = oracle.pack(L.T.copy(), abits, U)
    xin = oracle.pack(x.reshape(H * W, C), abits, U)          # packed HWC planes
    out = bs.bs_im2col_interleaved(planes_to_dev(xin), H, W, C, k, k, s, p)
    assert_equal(planes_to_numpy(out), want, "interleaved lowering")


def test_im2col_more_maps_than_grid_rows():
    """70000 one-plane images exceed the 65535 rows of the launch grid's second dimension, so workgroups walk
    several maps.  With a 1 x 1 kernel lowering is the identity on every image (checked on all of them), and a
    3 x 3 kernel is checked against the oracle on the first, one past the grid limit and the last image."""
    rng = np.random.default_rng(70000)
    B, H, W, C = 70000, 2, 2, 32
    x = rng.integers(0, 2, size=(B, H, W, C)).astype(np.int8)
    xp = bs.bs_pack_planes(dev(x.reshape(B * H * W, C)), 1, bs.BS_UNSIGNED)
    same = bs.bs_im2col_interleaved_batch(xp, B, H, W, C, 1, 1, 1, 0)
    assert torch.equal(same, xp), "1 x 1 lowering of a batch is the identity"
    low = planes_to_numpy(bs.bs_im2col_interleaved_batch(xp, B, H, W, C, 3, 3, 1, 1))   # [1][B * 4][words of 288 bits]
    for b in (0, 65535, 65536, B - 1):
        want = oracle.pack(oracle.im2col_plain(x[b], 3, 3, 1, 1).T.copy(), 1, U)
        assert_equal(low[:, 4 * b: 4 * b + 4], want, "image %d" % b)
