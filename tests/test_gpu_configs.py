"""GPU parity at the five benchmark configurations, full sizes, full outputs: every
int32 accumulator and every packed output word is compared with the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_1709_04060_amd as bs
from paper_1709_04060_amd import workloads
from gpu_util import assert_equal, dev, gemm_all_engines, gemm_threshold_all_engines, planes_to_numpy

pytestmark = pytest.mark.gpu
U, TC, BP = bs.BS_UNSIGNED, bs.BS_TWOS_COMPLEMENT, bs.BS_BIPOLAR


def test_cfg1_w1a2_tiny():
    d = workloads.cfg1_tiny()
    Wp = bs.bs_pack_planes(dev(d["W"]), 1, BP)
    Ap = bs.bs_pack_planes(dev(d["A"]), 2, U, depth_is_strided=True)
    assert_equal(planes_to_numpy(Wp), oracle.pack(d["W"], 1, oracle.BIPOLAR), "cfg1 W planes")
    assert_equal(planes_to_numpy(Ap), oracle.pack(d["A"].T, 2, oracle.UNSIGNED), "cfg1 A planes")
    C = bs.bs_gemm(Wp, BP, Ap, U, 256)
    assert_equal(C.cpu().numpy(), oracle.gemm(d["W"], d["A"]), "cfg1 C")


def test_cfg2_w2a2_4096_cubed():
    d = workloads.cfg2_square()
    Wp = bs.bs_pack_planes(dev(d["W"]), 2, TC)
    Ap = bs.bs_pack_planes(dev(d["A"]), 2, U, depth_is_strided=True)
    # the library's own choice, the AND-popcount kernel and both matrix-core kernels: one result, the oracle's
    assert_equal(gemm_all_engines(Wp, TC, Ap, U, 4096), oracle.gemm(d["W"], d["A"]), "cfg2 C")
    assert_equal(planes_to_numpy(Ap), oracle.pack(d["A"].T, 2, oracle.UNSIGNED), "cfg2 A planes")


def test_cfg3_fc6_fc7_chain():
    d = workloads.cfg3_fc_chain()
    W6p = bs.bs_pack_planes(dev(d["W6"]), 1, BP)
    W7p = bs.bs_pack_planes(dev(d["W7"]), 1, BP)
    xp = bs.bs_pack_planes(dev(d["x"]), 2, U, depth_is_strided=True)
    y6 = bs.bs_gemm_threshold(W6p, BP, xp, U, 9216, dev(d["thr6"]), 2)      # packed 2-bit, depth 4096
    y7 = bs.bs_gemm_threshold(W7p, BP, y6, U, 4096, dev(d["thr7"]), 2)      # consumed as the next activation
    C6 = oracle.gemm(d["W6"], d["x"])
    Y6 = oracle.threshold(C6, d["thr6"])
    assert_equal(planes_to_numpy(y6), oracle.threshold_pack(C6, d["thr6"], 2), "cfg3 fc6 output")
    C7 = oracle.gemm(d["W7"], Y6.astype(np.int8))
    assert_equal(planes_to_numpy(y7), oracle.threshold_pack(C7, d["thr7"], 2), "cfg3 fc7 output")
    # the thresholds are placed so that all four output levels occur
    assert len(np.unique(Y6)) == 4 and len(np.unique(oracle.threshold(C7, d["thr7"]))) == 4
    # unfused route gives the same planes
    c6 = bs.bs_gemm(W6p, BP, xp, U, 9216)
    assert_equal(c6.cpu().numpy(), C6, "cfg3 fc6 int32")
    assert_equal(planes_to_numpy(bs.bs_threshold_activate(c6, dev(d["thr6"]), 2)), planes_to_numpy(y6), "unfused")


def test_cfg4_conv2_lowered():
    d = workloads.cfg4_conv2()
    x, filt, s, p = d["x"], d["filt"], d["stride"], d["pad"]
    H, W, C = x.shape
    F, k = filt.shape[0], filt.shape[1]
    xp = bs.bs_pack_planes(dev(x.reshape(H * W, C)), 2, U)                  # packed HWC planes
    low = bs.bs_im2col_interleaved(xp, H, W, C, k, k, s, p)
    Kl = bs.bs_lowered_depth(C, k, k)
    assert Kl == 2400 and tuple(low.shape) == (2, 729, bs.bs_words_per_row(2400))
    Fp = bs.bs_pack_planes(dev(filt.reshape(F, -1)), 1, BP)                 # C = 96: no channel padding needed
    yp = gemm_threshold_all_engines(Fp, BP, low, U, Kl, dev(d["thr"]), 2)
    conv = oracle.conv_direct(x, filt, s, p)                                # [27][27][256], direct definition
    Cmat = conv.reshape(729, F).T.copy()
    assert_equal(yp, oracle.threshold_pack(Cmat, d["thr"], 2), "cfg4 packed output")
    assert_equal(gemm_all_engines(Fp, BP, low, U, Kl), Cmat, "cfg4 int32")
    L = oracle.im2col_plain(x, k, k, s, p)
    assert_equal(planes_to_numpy(low), oracle.pack(L.T.copy(), 2, oracle.UNSIGNED), "cfg4 lowered matrix")


@pytest.mark.parametrize("n", [1, 64, 1024, 8192])
def test_cfg5_w4a4_batch_sweep(n):
    d = workloads.cfg5_w4a4(n)
    Wp = bs.bs_pack_planes(dev(d["W"]), 4, TC)
    Ap = bs.bs_pack_planes(dev(d["A"]), 4, U, depth_is_strided=True)
    yp = gemm_threshold_all_engines(Wp, TC, Ap, U, 8192, dev(d["thr"]), 4)   # bit-serial and int8 matrix cores
    C = oracle.gemm(d["W"], d["A"])
    assert_equal(yp, oracle.threshold_pack(C, d["thr"], 4), "cfg5 packed output n=%d" % n)
    Y = oracle.threshold(C, d["thr"])
    assert len(np.unique(Y)) == 16                                          # all 16 levels occur
    if n <= 1024:
        assert_equal(gemm_all_engines(Wp, TC, Ap, U, 8192), C, "cfg5 int32 n=%d" % n)
