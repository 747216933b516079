"""The Python binding checks dtype, contiguity and shape of every tensor against the sizes it hands to the
library, on the host, before anything is called: a depth larger than the packed rows really hold would make
a kernel read past its buffers, and a wrong dtype or a strided view would give wrong numbers with BS_OK.
These tests need no GPU: they pass CPU tensors, so a call that got through validation would stop at the
"must be a GPU tensor" check, and every expected error must come before that."""
import pytest
import torch

import paper_1709_04060_amd as bs

U, TC, BP = bs.BS_UNSIGNED, bs.BS_TWOS_COMPLEMENT, bs.BS_BIPOLAR


def planes(bits, rows, depth, dtype=torch.int64):
    return torch.zeros((bits, rows, bs.bs_words_per_row(depth)), dtype=dtype)


def thr(M, obits, dtype=torch.int32):
    return torch.zeros((M, (1 << obits) - 1), dtype=dtype)


def test_valid_arguments_reach_the_device_check():
    """Correct shapes pass validation; the call then stops because the tensors are not on the GPU."""
    with pytest.raises(ValueError, match="GPU tensor"):
        bs.bs_gemm(planes(2, 8, 256), TC, planes(2, 4, 256), U, 256)
    with pytest.raises(ValueError, match="GPU tensor"):
        bs.bs_gemm_threshold(planes(1, 8, 100), BP, planes(2, 4, 100), U, 100, thr(8, 2), 2)
    with pytest.raises(ValueError, match="GPU tensor"):
        bs.bs_conv_threshold(planes(2, 25, 32), U, 5, 5, 32, planes(1, 16, 288), BP, 3, 3, 1, 1, thr(16, 2), 2)


@pytest.mark.parametrize("engine", [bs.BS_ENGINE_AUTO, bs.BS_ENGINE_BITSERIAL, bs.BS_ENGINE_DENSE_I8])
def test_gemm_depth_must_match_the_packed_rows(engine):
    Wp, Ap = planes(2, 8, 256), planes(2, 4, 256)
    with pytest.raises(ValueError, match="do not match depth"):
        bs.bs_gemm(Wp, TC, Ap, U, 512, engine=engine)            # K larger than the rows hold: an out-of-bounds read
    with pytest.raises(ValueError, match="do not match depth"):
        bs.bs_gemm(Wp, TC, planes(2, 4, 512), U, 256, engine=engine)
    with pytest.raises(ValueError, match="do not match depth"):
        bs.bs_gemm(Wp, TC, Ap, U, 0, engine=engine)
    with pytest.raises(ValueError, match="do not match depth"):
        bs.bs_gemm_threshold(Wp, TC, Ap, U, 1024, thr(8, 2), 2, engine=engine)
    with pytest.raises(ValueError, match="do not match depth"):
        bs.bs_gemm_topbits(Wp, TC, Ap, U, 1024, 1)


def test_plane_tensors_must_be_int64_contiguous_3d():
    good = planes(2, 4, 256)
    with pytest.raises(ValueError, match="int64"):
        bs.bs_gemm(planes(2, 8, 256, torch.int32), TC, good, U, 256)
    with pytest.raises(ValueError, match="contiguous"):
        bs.bs_gemm(planes(2, 16, 256)[:, ::2], TC, good, U, 256)
    with pytest.raises(ValueError, match="3-D"):
        bs.bs_gemm(planes(2, 8, 256)[0], TC, good, U, 256)
    with pytest.raises(ValueError, match="1..4 bit planes"):
        bs.bs_gemm(planes(5, 8, 256), TC, good, U, 256)


def test_thresholds_must_be_int32_of_the_right_shape():
    Wp, Ap = planes(1, 8, 128), planes(2, 4, 128)
    with pytest.raises(ValueError, match="int32"):
        bs.bs_gemm_threshold(Wp, BP, Ap, U, 128, thr(8, 2, torch.int64), 2)      # would be read as half as many rows
    with pytest.raises(ValueError, match=r"shape \[8\]\[3\]"):
        bs.bs_gemm_threshold(Wp, BP, Ap, U, 128, thr(8, 4), 2)
    with pytest.raises(ValueError, match=r"shape \[8\]\[3\]"):
        bs.bs_gemm_threshold(Wp, BP, Ap, U, 128, thr(7, 2), 2)
    with pytest.raises(ValueError, match="contiguous"):
        bs.bs_gemm_threshold(Wp, BP, Ap, U, 128, torch.zeros((8, 6), dtype=torch.int32)[:, ::2], 2)
    with pytest.raises(ValueError, match="obits"):
        bs.bs_gemm_threshold(Wp, BP, Ap, U, 128, thr(8, 2), 5)
    C = torch.zeros((8, 4), dtype=torch.int32)
    with pytest.raises(ValueError, match="int32"):
        bs.bs_threshold_activate(C, thr(8, 2, torch.int16), 2)
    with pytest.raises(ValueError, match="int32"):
        bs.bs_threshold_activate(C.to(torch.int64), thr(8, 2), 2)


def test_outputs_must_match():
    Wp, Ap = planes(2, 8, 256), planes(2, 4, 256)
    with pytest.raises(ValueError, match="int32"):
        bs.bs_gemm(Wp, TC, Ap, U, 256, out=torch.zeros((8, 4), dtype=torch.int64))
    with pytest.raises(ValueError, match=r"shape \[8\]\[4\]"):
        bs.bs_gemm(Wp, TC, Ap, U, 256, out=torch.zeros((8, 5), dtype=torch.int32))
    with pytest.raises(ValueError, match="unit column stride"):
        bs.bs_gemm(Wp, TC, Ap, U, 256, out=torch.zeros((4, 8), dtype=torch.int32).t())
    with pytest.raises(ValueError, match="must hold 2 planes"):
        bs.bs_gemm_threshold(Wp, TC, Ap, U, 256, thr(8, 2), 2, out=planes(3, 4, 8))
    with pytest.raises(ValueError, match="must hold 4 rows"):
        bs.bs_gemm_threshold(Wp, TC, Ap, U, 256, thr(8, 2), 2, out=planes(2, 5, 8))
    with pytest.raises(ValueError, match="do not match depth"):
        bs.bs_gemm_threshold(Wp, TC, Ap, U, 256, thr(8, 2), 2, out=planes(2, 4, 200))   # rows of M = 8 bits expected
    with pytest.raises(ValueError, match="must hold 8 rows"):
        bs.bs_pack_planes(torch.zeros((8, 100), dtype=torch.int8), 2, U, out=planes(2, 9, 100))
    with pytest.raises(ValueError, match="int8 or int32"):
        bs.bs_pack_planes(torch.zeros((8, 100), dtype=torch.int16), 2, U)


def test_convolution_and_pooling_geometry():
    x, Fp, t = planes(2, 25, 32), planes(1, 16, 288), thr(16, 2)
    with pytest.raises(ValueError, match="must hold 36 rows"):
        bs.bs_conv_threshold(x, U, 6, 6, 32, Fp, BP, 3, 3, 1, 1, t, 2)                  # map of 25 pixels passed as 6 x 6
    with pytest.raises(ValueError, match="do not match depth"):
        bs.bs_conv_threshold(x, U, 5, 5, 64, Fp, BP, 3, 3, 1, 1, t, 2)                  # more channels than packed
    with pytest.raises(ValueError, match="do not match depth"):
        bs.bs_conv_threshold(x, U, 5, 5, 32, planes(1, 16, 800), BP, 3, 3, 1, 1, t, 2)  # filters of another kernel size
    with pytest.raises(ValueError, match="geometry"):
        bs.bs_conv_threshold(x, U, 5, 5, 32, Fp, BP, 7, 7, 1, 0, t, 2)
    with pytest.raises(ValueError, match=r"shape \[16\]\[3\]"):
        bs.bs_conv_threshold(x, U, 5, 5, 32, Fp, BP, 3, 3, 1, 1, thr(15, 2), 2)
    with pytest.raises(ValueError, match="must hold 50 rows"):
        bs.bs_conv_threshold_batch(x, U, 2, 5, 5, 32, Fp, BP, 3, 3, 1, 1, t, 2)
    with pytest.raises(ValueError, match="must hold 36 rows"):
        bs.bs_im2col_interleaved(x, 6, 6, 32, 3, 3, 1, 1)
    with pytest.raises(ValueError, match="must hold 25 rows"):
        bs.bs_im2col_interleaved(x, 5, 5, 32, 3, 3, 1, 1, out=planes(2, 9, 288))
    with pytest.raises(ValueError, match="geometry"):
        bs.bs_maxpool_packed(x, 5, 5, 32, 6, 2)
    # convolution behind a pooling: 5 x 5 map, 2 x 2 / 1 windows -> 4 x 4 pooled map
    with pytest.raises(ValueError, match="GPU tensor"):
        bs.bs_pool_conv_threshold_batch(x, 1, 5, 5, 32, 2, 1, Fp, BP, 3, 3, 1, 1, t, 2)
    with pytest.raises(ValueError, match="pooling geometry"):
        bs.bs_pool_conv_threshold_batch(x, 1, 5, 5, 32, 6, 1, Fp, BP, 3, 3, 1, 1, t, 2)
    with pytest.raises(ValueError, match="convolution geometry"):
        bs.bs_pool_conv_threshold_batch(x, 1, 5, 5, 32, 2, 1, planes(1, 16, 800), BP, 5, 5, 1, 0, t, 2)   # 5 x 5 kernel on the 4 x 4 map
    with pytest.raises(ValueError, match="must hold 36 rows"):
        bs.bs_pool_conv_threshold_batch(x, 1, 6, 6, 32, 2, 1, Fp, BP, 3, 3, 1, 1, t, 2)
    with pytest.raises(ValueError, match="must hold 16 rows"):
        bs.bs_pool_conv_threshold_batch(x, 1, 5, 5, 32, 2, 1, Fp, BP, 3, 3, 1, 1, t, 2, out=planes(2, 25, 16))
    with pytest.raises(ValueError, match="must hold 36 rows"):
        bs.bs_maxpool_packed(x, 6, 6, 32, 3, 2)


def test_dense_operands():
    W, A = torch.zeros((8, 64), dtype=torch.int8), torch.zeros((4, 64), dtype=torch.int8)
    with pytest.raises(ValueError, match="shorter than the depth"):
        bs.bs_gemm_i8(W, A, 100)
    with pytest.raises(ValueError, match="int8"):
        bs.bs_gemm_i8(W.to(torch.uint8), A, 64)
    with pytest.raises(ValueError, match="depth-contiguous"):
        bs.bs_gemm_i8(torch.zeros((64, 8), dtype=torch.int8).t(), A, 64)
    with pytest.raises(ValueError, match="shorter than the depth"):
        bs.bs_gemm_fp4(W.to(torch.uint8), A.to(torch.uint8), 200)                      # 100 code bytes > 64
    with pytest.raises(ValueError, match="uint8"):
        bs.bs_gemm_fp4(W, A, 64)
    with pytest.raises(ValueError, match="int32"):
        bs.bs_gemm_i8_threshold(W, A, 64, thr(8, 2, torch.int64), 2)
    with pytest.raises(ValueError, match="do not match depth"):
        bs.bs_unpack_planes(planes(2, 8, 256), U, 1024)
    with pytest.raises(ValueError, match="shorter than the depth"):
        bs.bs_unpack_planes(planes(2, 8, 256), U, 256, out=torch.zeros((8, 128), dtype=torch.int8))
    with pytest.raises(ValueError, match="must hold 8 rows"):
        bs.bs_unpack_planes_fp4(planes(2, 8, 256), U, 256, out=torch.zeros((9, 128), dtype=torch.uint8))
    with pytest.raises(ValueError, match="GPU tensor"):
        bs.bs_gemm_i8(W, A, 64)


def test_engine_choice_respects_the_dense_engines_depth_limits():
    """bs_choose_engine never names an engine whose kernel would refuse the call: the fp4 kernel needs
    K (2^wbits - 1) (2^abits - 1) < 2^24, both dense kernels K < 2^30."""
    E = bs.bs_choose_engine
    assert E(2, TC, 2, U, 4096, 4096, 4096) == bs.BS_ENGINE_DENSE_FP4
    assert E(2, TC, 2, U, 4096, 4096, 1864136) == bs.BS_ENGINE_DENSE_I8      # 3 * 3 * K >= 2^24: int32 accumulation instead
    assert E(2, TC, 2, U, 4096, 4096, 1864135) == bs.BS_ENGINE_DENSE_FP4
    assert E(1, BP, 1, BP, 4096, 4096, 1 << 24) == bs.BS_ENGINE_DENSE_I8
    assert E(1, BP, 1, BP, 4096, 4096, (1 << 24) - 1) == bs.BS_ENGINE_DENSE_FP4
    assert E(1, BP, 4, U, 4096, 4096, 1 << 30) == bs.BS_ENGINE_BITSERIAL
    assert E(1, BP, 4, U, 4096, 4096, 1 << 20) == bs.BS_ENGINE_DENSE_I8
