"""Pins for direct convolution and plain lowering (O3, Sec. 3 and 3.2)."""
import numpy as np
import pytest

import oracle


@pytest.mark.parametrize("H,W,C,F,k,s,p", [(5, 6, 3, 4, 3, 1, 1), (7, 7, 8, 5, 5, 1, 2), (9, 8, 4, 3, 3, 2, 0),
                                           (6, 6, 2, 2, 1, 1, 0), (8, 9, 5, 3, 3, 2, 1)])
def test_direct_equals_lowering_then_gemm(H, W, C, F, k, s, p):
    rng = np.random.default_rng(H * W + C)
    x = rng.integers(0, 4, size=(H, W, C)).astype(np.int8)
    filt = (2 * rng.integers(0, 2, size=(F, k, k, C)) - 1).astype(np.int8)
    out = oracle.conv_direct(x, filt, s, p)
    OH, OW = oracle.conv_out_size(H, W, k, k, s, p)
    assert out.shape == (OH, OW, F)
    L = oracle.im2col_plain(x, k, k, s, p)
    via = (filt.reshape(F, -1).astype(np.int64) @ L.astype(np.int64))       # library matmul
    assert np.array_equal(out.reshape(OH * OW, F).T.astype(np.int64), via)
    # and a direct Python evaluation of a few outputs
    for (oh, ow, f) in [(0, 0, 0), (OH - 1, OW - 1, F - 1), (OH // 2, OW // 2, F // 2)]:
        acc = 0
        for kh in range(k):
            for kw in range(k):
                ih, iw = oh * s + kh - p, ow * s + kw - p
                if 0 <= ih < H and 0 <= iw < W:
                    acc += int(np.dot(filt[f, kh, kw].astype(np.int64), x[ih, iw].astype(np.int64)))
        assert int(out[oh, ow, f]) == acc


def test_one_by_one_kernel_is_a_gemm():
    rng = np.random.default_rng(5)
    x = rng.integers(0, 4, size=(4, 5, 7)).astype(np.int8)
    filt = rng.integers(-2, 2, size=(6, 1, 1, 7)).astype(np.int8)
    out = oracle.conv_direct(x, filt, 1, 0)
    ref = oracle.gemm(filt.reshape(6, 7), x.reshape(20, 7).T.copy())
    assert np.array_equal(out.reshape(20, 6).T, ref)


def test_all_ones_counts_in_image_taps():
    H = W = 6; C = 3; k = 5; p = 2
    x = np.ones((H, W, C), dtype=np.int8)
    filt = np.ones((2, k, k, C), dtype=np.int8)
    out = oracle.conv_direct(x, filt, 1, p)
    for oh in range(H):
        for ow in range(W):
            nh = sum(1 for kh in range(k) if 0 <= oh + kh - p < H)
            nw = sum(1 for kw in range(k) if 0 <= ow + kw - p < W)
            assert (out[oh, ow] == nh * nw * C).all()


def test_im2col_row_order_is_kh_kw_c():
    x = np.arange(3 * 3 * 2, dtype=np.int8).reshape(3, 3, 2)
    L = oracle.im2col_plain(x, 2, 2, 1, 0)
    assert L.shape == (8, 4)
    # column 0 = output pixel (0,0): taps (0,0),(0,1),(1,0),(1,1), channels fastest
    assert list(L[:, 0]) == [0, 1, 2, 3, 6, 7, 8, 9]
    assert list(L[:, 3]) == [8, 9, 10, 11, 14, 15, 16, 17]


@pytest.mark.parametrize("H,W,C,k,s", [(27, 27, 5, 3, 2), (13, 13, 7, 3, 2), (8, 9, 3, 2, 2), (6, 6, 2, 3, 1)])
def test_maxpool_against_library_filter(H, W, C, k, s):
    """oracle.maxpool against numpy's sliding-window view and scipy's maximum_filter."""
    from scipy.ndimage import maximum_filter
    rng = np.random.default_rng(H + W + C)
    Y = rng.integers(0, 4, size=(H, W, C)).astype(np.uint8)
    got = oracle.maxpool(Y, k, s)
    OH, OW = (H - k) // s + 1, (W - k) // s + 1
    assert got.shape == (OH, OW, C)
    view = np.lib.stride_tricks.sliding_window_view(Y, (k, k), axis=(0, 1))     # [H-k+1][W-k+1][C][k][k]
    ref = view.max(axis=(-1, -2))[::s, ::s, :]
    if k % 2 == 1:  # scipy's centred filter: window at centre i covers i - k//2 .. i + k//2
        full = maximum_filter(Y, size=(k, k, 1), mode="constant", cval=0)
        assert np.array_equal(full[k // 2: k // 2 + (OH - 1) * s + 1: s, k // 2: k // 2 + (OW - 1) * s + 1: s, :], ref)
    assert np.array_equal(got, ref)
    # monotone: pooling commutes with thresholding of the underlying accumulators
    C32 = rng.integers(-100, 100, size=(H, W, C)).astype(np.int32)
    thr = np.sort(rng.integers(-80, 80, size=(C, 3)), axis=1).astype(np.int32)
    Yt = oracle.threshold(C32.reshape(-1, C).T, thr).T.reshape(H, W, C)
    pooled_acc = oracle.maxpool(C32, k, s)
    assert np.array_equal(oracle.maxpool(Yt, k, s),
                          oracle.threshold(pooled_acc.reshape(-1, C).T, thr).T.reshape(OH, OW, C))


def test_maxpool_closed_forms():
    Y = np.full((7, 7, 3), 2, dtype=np.uint8)
    assert (oracle.maxpool(Y, 3, 2) == 2).all()
    Y[3, 3, 1] = 3
    out = oracle.maxpool(Y, 3, 2)                 # windows cover 0..2, 2..4, 4..6: pixel 3 lies in window 1 only
    assert out.shape == (3, 3, 3)
    want = np.full((3, 3, 3), 2); want[1, 1, 1] = 3
    assert np.array_equal(out, want)
    Y[4, 2, 0] = 3                                # pixel (4, 2) lies in windows (1, 0), (1, 1), (2, 0), (2, 1)
    want[1:3, 0:2, 0] = 3
    assert np.array_equal(oracle.maxpool(Y, 3, 2), want)
