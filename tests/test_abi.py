"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
the header declares, its host helpers agree with the documented format, and argument
errors are caught before anything is launched."""
import ctypes
import os
import re

import pytest

import oracle
import paper_1709_04060_amd as bs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "bsgemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bs_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = bs.load_library()
    names = declared_functions()
    assert set(names) == set(bs.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_host_helpers():
    for k in (1, 63, 64, 65, 128, 129, 2400, 4096, 9216):
        assert bs.bs_words_per_row(k) == oracle.words_per_row(k)
    assert bs.bs_words_per_row(0) == 0
    assert bs.bs_lowered_depth(96, 5, 5) == 2400
    assert bs.bs_lowered_depth(3, 3, 3) == 9 * 32
    assert bs.bs_version() >= 100
    assert bs.status_string(0) == "ok" and "overflow" in bs.status_string(-4)


def test_argument_errors_are_rejected_on_the_host():
    lib = bs.load_library()
    p = 0x1000  # a fake, aligned, never dereferenced address: every call below must fail before launch
    assert lib.bs_gemm(None, 1, 0, p, 1, 0, 4, 4, 64, p, 4, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_gemm(p, 0, 0, p, 1, 0, 4, 4, 64, p, 4, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_gemm(p, 5, 0, p, 1, 0, 4, 4, 64, p, 4, None) == bs.BS_ERR_UNSUPPORTED
    assert lib.bs_gemm(p, 2, bs.BS_BIPOLAR, p, 1, 0, 4, 4, 64, p, 4, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_gemm(p, 1, 0, p, 1, 0, 0, 4, 64, p, 4, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_gemm(p, 1, 0, p, 1, 0, 4, 4, 64, p, 3, None) == bs.BS_ERR_INVALID_ARG      # ldc < N
    assert lib.bs_gemm(p + 8, 1, 0, p, 1, 0, 4, 4, 64, p, 4, None) == bs.BS_ERR_ALIGNMENT
    assert lib.bs_gemm(p, 4, 1, p, 4, 0, 4, 4, 1 << 23, p, 4, None) == bs.BS_ERR_OVERFLOW_RISK
    assert lib.bs_gemm_threshold(p, 1, 0, p, 1, 0, 4, 4, 64, None, 2, p, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_gemm_threshold(p, 1, 0, p, 1, 0, 4, 4, 64, p, 5, p, None) == bs.BS_ERR_UNSUPPORTED
    assert lib.bs_pack_planes(p, 7, 4, 64, 64, 0, 1, 0, p, None) == bs.BS_ERR_INVALID_ARG      # dtype
    assert lib.bs_pack_planes(p, 0, 4, 64, 32, 0, 1, 0, p, None) == bs.BS_ERR_INVALID_ARG      # ld < depth
    assert lib.bs_pack_planes(p, 0, 4, 64, 64, 0, 2, bs.BS_BIPOLAR, p, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_threshold_activate(p, 4, 4, 4, p, 0, p, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_im2col_interleaved(p, 2, 3, 3, 8, 7, 7, 1, 0, p, None) == bs.BS_ERR_INVALID_ARG  # kernel > image
    assert lib.bs_im2col_interleaved(p, 2, 3, 3, 8, 3, 3, 0, 0, p, None) == bs.BS_ERR_INVALID_ARG  # stride 0
