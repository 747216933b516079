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
    # |C| <= K max|w| max|a| must stay below 2^31 (refused cases only: an accepted call would launch on the fake address)
    assert lib.bs_gemm(p, 4, 1, p, 4, 0, 4, 4, 17895698, p, 4, None) == bs.BS_ERR_OVERFLOW_RISK          # 8 * 15 * K
    assert lib.bs_gemm(p, 4, 0, p, 4, 0, 4, 4, 9544372, p, 4, None) == bs.BS_ERR_OVERFLOW_RISK           # 15 * 15 * K
    assert lib.bs_gemm(p, 2, 1, p, 2, 0, 4, 4, 357913942, p, 4, None) == bs.BS_ERR_OVERFLOW_RISK         # 2 * 3 * K
    assert lib.bs_gemm(p, 1, 2, p, 2, 0, 4, 4, 715827883, p, 4, None) == bs.BS_ERR_OVERFLOW_RISK         # 1 * 3 * K
    assert lib.bs_gemm(p, 1, 2, p, 1, 2, 4, 4, 1 << 31, p, 4, None) == bs.BS_ERR_OVERFLOW_RISK
    assert lib.bs_gemm(p, 1, 0, p, 1, 0, 4, 4, (1 << 31) - 1, p, 4, None) == bs.BS_ERR_OVERFLOW_RISK    # a result could be INT_MAX
    # the approximate mode sums a subset of the plane pairs: bounded by the unsigned ranges, 15 * 15 * K
    assert lib.bs_gemm_topbits(p, 4, 1, p, 4, 0, 4, 4, 9544372, 3, p, 4, None) == bs.BS_ERR_OVERFLOW_RISK
    # engines: unknown value; the fp4 matrix-core kernel takes operands of at most two bits and 9 K < 2^24 for two planes each
    assert lib.bs_gemm_on(7, p, 1, 0, p, 1, 0, 4, 4, 64, p, 4, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_gemm_on(bs.BS_ENGINE_DENSE_FP4, p, 3, 1, p, 2, 0, 4, 4, 64, p, 4, None) == bs.BS_ERR_UNSUPPORTED
    assert lib.bs_gemm_on(bs.BS_ENGINE_DENSE_FP4, p, 2, 1, p, 2, 0, 4, 4, 1864136, p, 4, None) == bs.BS_ERR_UNSUPPORTED   # 9 K >= 2^24
    assert lib.bs_gemm_threshold_on(bs.BS_ENGINE_DENSE_I8, p, 1, 2, p, 1, 2, 4, 4, 1 << 30, p, 1, p, None) == bs.BS_ERR_UNSUPPORTED
    assert lib.bs_gemm_threshold(p, 1, 0, p, 1, 0, 4, 4, 64, None, 2, p, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_gemm_threshold(p, 1, 0, p, 1, 0, 4, 4, 64, p, 5, p, None) == bs.BS_ERR_UNSUPPORTED
    assert lib.bs_pack_planes(p, 7, 4, 64, 64, 0, 1, 0, p, None) == bs.BS_ERR_INVALID_ARG      # dtype
    assert lib.bs_pack_planes(p, 0, 4, 64, 32, 0, 1, 0, p, None) == bs.BS_ERR_INVALID_ARG      # ld < depth
    assert lib.bs_pack_planes(p, 0, 4, 64, 64, 0, 2, bs.BS_BIPOLAR, p, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_threshold_activate(p, 4, 4, 4, p, 0, p, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_im2col_interleaved(p, 2, 3, 3, 8, 7, 7, 1, 0, p, None) == bs.BS_ERR_INVALID_ARG  # kernel > image
    assert lib.bs_im2col_interleaved(p, 2, 3, 3, 8, 3, 3, 0, 0, p, None) == bs.BS_ERR_INVALID_ARG  # stride 0


def test_argument_errors_of_the_later_entry_points():
    lib = bs.load_library()
    p = 0x1000
    U, BP = bs.BS_UNSIGNED, bs.BS_BIPOLAR
    # fused convolution: bipolar activations cannot be zero-padded, kernel larger than image, lowered depth too large
    assert lib.bs_conv_threshold(p, 1, BP, 8, 8, 32, p, 1, BP, 16, 3, 3, 1, 1, p, 2, p, None) == bs.BS_ERR_UNSUPPORTED
    assert lib.bs_conv_threshold(p, 2, U, 3, 3, 32, p, 1, BP, 16, 5, 5, 1, 0, p, 2, p, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_conv_threshold(p, 2, U, 64, 64, 4096, p, 1, BP, 16, 7, 7, 1, 3, p, 2, p, None) == bs.BS_ERR_UNSUPPORTED
    assert lib.bs_conv_threshold(None, 2, U, 8, 8, 32, p, 1, BP, 16, 3, 3, 1, 1, p, 2, p, None) == bs.BS_ERR_INVALID_ARG
    # pooling window larger than the map
    assert lib.bs_maxpool_packed(p, 2, 2, 2, 32, 3, 2, p, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_maxpool_packed(p, 5, 8, 8, 32, 3, 2, p, None) == bs.BS_ERR_UNSUPPORTED
    # convolution behind a pooling: window of 1..3 inside the map, a kernel that fits the POOLED map
    pc = lib.bs_pool_conv_threshold_batch   # in, abits, B, H, W, C, pool_k, pool_stride, Fp, wbits, wfmt, F, kh, kw, stride, pad, thr, obits, Yp, stream
    assert pc(p, 2, 1, 13, 13, 64, 0, 2, p, 1, BP, 16, 3, 3, 1, 1, p, 2, p, None) == bs.BS_ERR_INVALID_ARG
    assert pc(p, 2, 1, 13, 13, 64, 3, 0, p, 1, BP, 16, 3, 3, 1, 1, p, 2, p, None) == bs.BS_ERR_INVALID_ARG
    assert pc(p, 2, 1, 2, 2, 64, 3, 2, p, 1, BP, 16, 1, 1, 1, 0, p, 2, p, None) == bs.BS_ERR_INVALID_ARG
    assert pc(p, 2, 1, 13, 13, 64, 4, 2, p, 1, BP, 16, 3, 3, 1, 1, p, 2, p, None) == bs.BS_ERR_UNSUPPORTED
    assert pc(p, 2, 1, 13, 13, 64, 3, 2, p, 1, BP, 16, 7, 7, 1, 0, p, 2, p, None) == bs.BS_ERR_INVALID_ARG      # pooled map is 6 x 6
    assert pc(p, 2, 1, 13, 13, 64, 3, 2, None, 1, BP, 16, 3, 3, 1, 1, p, 2, p, None) == bs.BS_ERR_INVALID_ARG
    assert pc(p, 2, 1, 13, 13, 64, 3, 2, p, 1, BP, 16, 3, 3, 1, 1, p, 2, p + 8, None) == bs.BS_ERR_ALIGNMENT
    # dense engine: leading dimensions must be multiples of 16 and >= K; depth bound
    assert lib.bs_gemm_i8(p, 24, p, 32, 4, 4, 20, p, 4, None) == bs.BS_ERR_ALIGNMENT
    assert lib.bs_gemm_i8(p, 16, p, 32, 4, 4, 20, p, 4, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_gemm_i8(p, 1 << 17, p, 1 << 17, 4, 4, 1 << 17, p, 4, None) == bs.BS_ERR_OVERFLOW_RISK
    assert lib.bs_gemm_i8_threshold(p, 32, p, 32, 4, 4, 20, None, 2, p, None) == bs.BS_ERR_INVALID_ARG
    assert lib.bs_unpack_planes(p, 2, U, 4, 20, p, 16, None) == bs.BS_ERR_INVALID_ARG          # ld < 32
    assert lib.bs_unpack_planes(p, 2, BP, 4, 20, p, 32, None) == bs.BS_ERR_INVALID_ARG         # bipolar needs 1 bit


def test_oracle_c_part_is_clean_under_sanitizers(tmp_path):
    """The oracle's C file built with AddressSanitizer + UBSan (host only) and driven through a
    small main(): out-of-bounds or undefined behaviour in the reference would poison every parity claim."""
    import subprocess
    import textwrap
    main_c = tmp_path / "main.c"
    main_c.write_text(textwrap.dedent("""
        #include <stdint.h>
        #include <stdlib.h>
        #include <stdio.h>
        void oracle_gemm_i8(const int8_t*, const int8_t*, int32_t*, int64_t, int64_t, int64_t);
        void oracle_pack(const int32_t*, int64_t, int64_t, int, int, uint64_t*, int64_t);
        void oracle_bitserial_gemm(const uint64_t*, int, int, const uint64_t*, int, int, int64_t*, int64_t, int64_t, int64_t, int64_t, int64_t);
        void oracle_conv_direct(const int8_t*, const int8_t*, int32_t*, int, int, int, int, int, int, int, int);
        void oracle_im2col_plain(const int8_t*, int8_t*, int, int, int, int, int, int, int);
        int main(void) {
            enum { M = 7, K = 130, N = 5, S = 4 };
            int8_t *W = malloc(M * K), *A = malloc(K * N); int32_t *C = malloc(sizeof(int32_t) * M * N);
            int32_t *Wi = malloc(sizeof(int32_t) * M * K), *Ai = malloc(sizeof(int32_t) * N * K);
            for (int i = 0; i < M * K; ++i) { W[i] = (int8_t)(i % 4 - 2); Wi[i] = W[i]; }
            for (int k = 0; k < K; ++k) for (int n = 0; n < N; ++n) { A[k * N + n] = (int8_t)((k + n) % 4); Ai[n * K + k] = A[k * N + n]; }
            oracle_gemm_i8(W, A, C, M, K, N);
            uint64_t *Wp = malloc(8 * 2 * M * S), *Ap = malloc(8 * 2 * N * S); int64_t *R = malloc(8 * M * N);
            oracle_pack(Wi, M, K, 2, 1, Wp, S); oracle_pack(Ai, N, K, 2, 0, Ap, S);
            oracle_bitserial_gemm(Wp, 2, 1, Ap, 2, 0, R, M, N, S, S, S);
            for (int i = 0; i < M * N; ++i) if (R[i] != C[i]) { puts("mismatch"); return 1; }
            int8_t *img = calloc(6 * 6 * 3, 1), *f = calloc(4 * 3 * 3 * 3, 1); int32_t *o = malloc(4 * 6 * 6 * 4);
            int8_t *L = malloc(27 * 36);
            oracle_conv_direct(img, f, o, 6, 6, 3, 4, 3, 3, 1, 1);
            oracle_im2col_plain(img, L, 6, 6, 3, 3, 3, 1, 1);
            free(W); free(A); free(C); free(Wi); free(Ai); free(Wp); free(Ap); free(R); free(img); free(f); free(o); free(L);
            puts("ok"); return 0;
        }"""))
    exe = tmp_path / "oracle_asan"
    src = os.path.join(ROOT, "oracle", "bs_oracle.c")
    # the sanitizer runtimes are linked statically, so no preload order matters
    subprocess.check_call(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-static-libasan", "-static-libubsan", "-std=c11", "-o", str(exe), str(main_c), src])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0 and "ok" in out.stdout, out.stdout + out.stderr


def test_engine_choice_rules():
    """bs_choose_engine (host-only): the fixed rules and the monotone behaviour of the fitted model."""
    E = bs.bs_choose_engine
    U, TC, BP = bs.BS_UNSIGNED, bs.BS_TWOS_COMPLEMENT, bs.BS_BIPOLAR
    BSER, I8, FP4 = bs.BS_ENGINE_BITSERIAL, bs.BS_ENGINE_DENSE_I8, bs.BS_ENGINE_DENSE_FP4
    # few columns: weights are streamed once, the packed form always wins
    for n in (1, 2, 4):
        assert E(4, TC, 4, U, 8192, n, 8192) == BSER and E(2, TC, 2, U, 8192, n, 8192) == BSER
    # invalid arguments fall back to the bit-serial engine
    assert E(0, U, 2, U, 64, 64, 64) == BSER and E(2, U, 5, U, 64, 64, 64) == BSER and E(2, U, 2, U, 0, 64, 64) == BSER
    assert E(2, BP, 2, U, 4096, 4096, 4096) == BSER
    # large compute-bound products go to the matrix cores: fp4 where every value is an E2M1 number, else int8
    assert E(4, TC, 4, U, 8192, 8192, 8192) == I8
    assert E(2, TC, 2, U, 4096, 4096, 4096) == FP4
    assert E(1, BP, 2, U, 4096, 4096, 4096) == FP4
    assert E(3, TC, 2, U, 4096, 4096, 4096) == I8      # the plane loader's fp4 path takes at most two planes
    assert E(3, U, 2, U, 4096, 4096, 4096) == I8       # 5 and 7 are not E2M1 numbers
    # small layers stay bit-serial
    assert E(1, BP, 1, BP, 256, 256, 1024) == BSER
    assert E(1, BP, 2, U, 256, 729, 2400) == BSER      # the conv2 layer of the paper's AlexNet at batch 1
    # once a dense engine is chosen, more plane pairs never switch back
    for (m, n, k) in [(1024, 1024, 4096), (4096, 256, 4096), (256, 4096, 1024)]:
        seen = False
        for (w, a) in [(1, 1), (1, 2), (2, 2), (2, 4), (4, 4)]:
            d = E(w, TC, a, U, m, n, k) != BSER
            assert d or not seen
            seen = seen or d
