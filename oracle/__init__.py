"""CPU oracle for the bit-serial GEMM hot path -- TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct statement of what the hot path computes,
written from the paper's definitions.  It is independent of the HIP library:
no shared kernels, headers, helpers, tables or pre/post-processing, and it
imports nothing from the product package.  Only ``tests/``, the smoke check and
the benchmark's ``cpu_baseline`` leg may use it.

The heavy loops live in ``bs_oracle.c`` (plain C, built here with gcc and
loaded through ctypes); the thin numpy parts are in this file.  Every function
cites the passage of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bs_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

UNSIGNED, TWOS_COMPLEMENT, BIPOLAR = 0, 1, 2


# ISA level x86-64-v3 (AVX2), not -march=native: the library is built where there is no GPU and travels to the box
# that runs it.  Timings of the oracle therefore understate what the host could do with its own widest vectors.
COMPILE_FLAGS = ["-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall"]


def build(force: bool = False) -> str:
    """Compile bs_oracle.c into liboracle.so (gcc, OpenMP).  Portable ISA level
    (no -march=native) so that a library built on one host runs on another."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc"] + COMPILE_FLAGS + ["-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.oracle_gemm_i8.argtypes = [vp, vp, vp, i64, i64, i64]
        lib.oracle_gemm_i8.restype = None
        lib.oracle_dot_i8.argtypes = [vp, vp, i64, i64, i64, i64]
        lib.oracle_dot_i8.restype = ctypes.c_int64
        lib.oracle_pack.argtypes = [vp, i64, i64, i32, i32, vp, i64]
        lib.oracle_pack.restype = None
        lib.oracle_bitserial_gemm.argtypes = [vp, i32, i32, vp, i32, i32, vp, i64, i64, i64, i64, i64]
        lib.oracle_bitserial_gemm.restype = None
        lib.oracle_bitserial_gemm_from.argtypes = [vp, i32, i32, vp, i32, i32, vp, i64, i64, i64, i64, i64, i32]
        lib.oracle_bitserial_gemm_from.restype = None
        lib.oracle_conv_direct.argtypes = [vp, vp, vp] + [i32] * 8
        lib.oracle_conv_direct.restype = None
        lib.oracle_im2col_plain.argtypes = [vp, vp] + [i32] * 7
        lib.oracle_im2col_plain.restype = None
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    """Threads the OpenMP loops of the C part will use."""
    return int(_load().oracle_num_threads())


def words_per_row(depth: int) -> int:
    """Row stride, in 64-bit words, of a packed plane: ceil(depth/64) rounded up
    to an even count (rows start on 16-byte boundaries).  Part of the packed
    format that crosses the library boundary; restated here on purpose."""
    return 2 * ((int(depth) + 127) // 128)


# --------------------------------------------------------------------------- O1
def gemm(W: np.ndarray, A: np.ndarray) -> np.ndarray:
    """C = W . A by the plain definition (Sec. 3.1).  W [M][K], A [K][N] hold
    logical values as int8; result int32 [M][N]."""
    W = np.ascontiguousarray(W, dtype=np.int8)
    A = np.ascontiguousarray(A, dtype=np.int8)
    M, K = W.shape
    K2, N = A.shape
    assert K == K2
    C = np.empty((M, N), dtype=np.int32)
    _load().oracle_gemm_i8(_p(W), _p(A), _p(C), M, K, N)
    return C


def dot(W: np.ndarray, A: np.ndarray, m: int, n: int) -> int:
    """One element C[m][n] of the same product, in 64-bit (sampled checks)."""
    assert W.dtype == np.int8 and A.dtype == np.int8 and W.flags.c_contiguous and A.flags.c_contiguous
    M, K = W.shape
    _, N = A.shape
    return int(_load().oracle_dot_i8(_p(W), _p(A), int(m), int(n), K, N))


# --------------------------------------------------------------------------- O4
def pack(X: np.ndarray, bits: int, fmt: int) -> np.ndarray:
    """Bit planes of X [rows][depth] (logical values): uint64 [bits][rows][stride],
    bit b of word d <-> depth index 64 d + b, zero beyond depth (Sec. 3.1, Alg. 1).
    Encodings: unsigned v; two's complement v mod 2^bits; bipolar (v + 1) / 2."""
    X = np.ascontiguousarray(X, dtype=np.int32)
    rows, depth = X.shape
    stride = words_per_row(depth)
    planes = np.empty((bits, rows, stride), dtype=np.uint64)
    _load().oracle_pack(_p(X), rows, depth, bits, fmt, _p(planes), stride)
    return planes


# ------------------------------------------------------------------------ O1b(i)
def bitserial_gemm(Wp: np.ndarray, wsigned: bool, Ap: np.ndarray, asigned: bool) -> np.ndarray:
    """Algorithms 1 and 2 step by step on packed planes Wp [w][rows][stride],
    Ap [a][cols][stride]: sum over plane pairs of sgn * 2^(i+j) * popcount(AND).
    int64 result [rows][cols]."""
    Wp = np.ascontiguousarray(Wp, dtype=np.uint64)
    Ap = np.ascontiguousarray(Ap, dtype=np.uint64)
    w, rows, ws = Wp.shape
    a, cols, as_ = Ap.shape
    assert ws == as_
    res = np.empty((rows, cols), dtype=np.int64)
    _load().oracle_bitserial_gemm(_p(Wp), w, int(bool(wsigned)), _p(Ap), a, int(bool(asigned)),
                                  _p(res), rows, cols, ws, ws, as_)
    return res


def bitserial_gemm_topbits(Wp: np.ndarray, wsigned: bool, Ap: np.ndarray, asigned: bool, min_shift: int) -> np.ndarray:
    """Alg. 2 restricted to the plane pairs with i + j >= min_shift (approximation from the
    higher-order bits, named as future work in the paper's conclusion).  int64 [rows][cols]."""
    Wp = np.ascontiguousarray(Wp, dtype=np.uint64)
    Ap = np.ascontiguousarray(Ap, dtype=np.uint64)
    w, rows, ws = Wp.shape
    a, cols, as_ = Ap.shape
    res = np.empty((rows, cols), dtype=np.int64)
    _load().oracle_bitserial_gemm_from(_p(Wp), w, int(bool(wsigned)), _p(Ap), a, int(bool(asigned)),
                                       _p(res), rows, cols, ws, ws, as_, int(min_shift))
    return res


def _popcount_rows(P: np.ndarray) -> np.ndarray:
    """popcount over the last axis of a uint64 array, one bit at a time."""
    bits = np.unpackbits(np.ascontiguousarray(P).view(np.uint8), axis=-1)
    return bits.sum(axis=-1, dtype=np.int64)


def bipolar_weight_gemm(Bp: np.ndarray, Ap: np.ndarray) -> np.ndarray:
    """O1b(ii): +-1 weights (w = 2b - 1, b the packed bit) times unsigned a-bit
    activations:  C = sum_j 2^j * (2 popcount(B & A[j]) - popcount(A[j])).
    Follows from substituting w = 2b - 1 in the plane identity of Sec. 3.1."""
    a = Ap.shape[0]
    rows, cols = Bp.shape[1], Ap.shape[1]
    C = np.zeros((rows, cols), dtype=np.int64)
    for j in range(a):
        pa = _popcount_rows(Ap[j])                                  # [cols]
        for r in range(rows):
            C[r] += (1 << j) * (2 * _popcount_rows(Bp[0, r][None, :] & Ap[j]) - pa)
    return C


def bipolar_xor_gemm(Bw: np.ndarray, Ba: np.ndarray, K: int) -> np.ndarray:
    """O1b(iii): +-1 times +-1 via the binary dot product of prior work cited in
    Sec. 3.1:  dot = K - 2 popcount(Bw XOR Ba) over the true depth K (padding
    bits are zero in both operands, so they never differ)."""
    rows, cols = Bw.shape[1], Ba.shape[1]
    C = np.zeros((rows, cols), dtype=np.int64)
    for r in range(rows):
        C[r] = K - 2 * _popcount_rows(Bw[0, r][None, :] ^ Ba[0])
    return C


# --------------------------------------------------------------------------- O2
def threshold(C: np.ndarray, thr: np.ndarray) -> np.ndarray:
    """Successive thresholding T(x, t) of Sec. 2.1.1 by counting: the number of
    thresholds that x is greater than or equal to.  C [M][N] (any real dtype),
    thr [M][T] per output row; result uint8 [M][N] in 0..T."""
    C = np.asarray(C)
    thr = np.asarray(thr)
    Y = np.zeros(C.shape, dtype=np.uint8)
    for i in range(thr.shape[1]):
        Y += (C >= thr[:, i][:, None]).astype(np.uint8)
    return Y


def threshold_pack(C: np.ndarray, thr: np.ndarray, obits: int) -> np.ndarray:
    """Thresholded activations as channel-interleaved bit planes: plane p of
    column n holds bit p of Y[m][n] for every output row (channel) m, packed along
    m like any other depth (Sec. 3.2: each pixel holds one bit position of all
    channels).  uint64 [obits][N][words_per_row(M)]."""
    assert thr.shape[1] == (1 << obits) - 1
    Y = threshold(C, thr)
    return pack(Y.T.astype(np.int32), obits, UNSIGNED)


# --------------------------------------------------------------------------- O3
def conv_out_size(H, W, KH, KW, s, p):
    return (H + 2 * p - KH) // s + 1, (W + 2 * p - KW) // s + 1


def conv_direct(x: np.ndarray, filt: np.ndarray, stride: int, pad: int) -> np.ndarray:
    """Convolution by its direct definition on x [H][W][C], filt [F][KH][KW][C];
    int32 [OH][OW][F].  Out-of-image taps are 0."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    filt = np.ascontiguousarray(filt, dtype=np.int8)
    H, W, C = x.shape
    F, KH, KW, C2 = filt.shape
    assert C == C2
    OH, OW = conv_out_size(H, W, KH, KW, stride, pad)
    out = np.empty((OH, OW, F), dtype=np.int32)
    _load().oracle_conv_direct(_p(x), _p(filt), _p(out), H, W, C, F, KH, KW, stride, pad)
    return out


def im2col_plain(x: np.ndarray, KH: int, KW: int, stride: int, pad: int) -> np.ndarray:
    """Plain lowering (Sec. 3.2) of x [H][W][C] to L [(kh KW + kw) C + c][oh OW + ow]."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    H, W, C = x.shape
    OH, OW = conv_out_size(H, W, KH, KW, stride, pad)
    L = np.empty((KH * KW * C, OH * OW), dtype=np.int8)
    _load().oracle_im2col_plain(_p(x), _p(L), H, W, C, KH, KW, stride, pad)
    return L


def maxpool(Y: np.ndarray, k: int, stride: int) -> np.ndarray:
    """Max pooling of a few-bit activation map Y [H][W][C] by its definition: the largest
    value in each k x k window, windows stride apart, no padding.  Thresholding is
    monotone, so pooling the thresholded codes equals thresholding the pooled
    accumulators; the paper keeps pooling outside its hot path (Sec. 4.2), here it joins
    the packed layers into a chain.  [OH][OW][C], OH = (H - k) // stride + 1."""
    Y = np.asarray(Y)
    H, W, C = Y.shape
    OH, OW = (H - k) // stride + 1, (W - k) // stride + 1
    out = np.empty((OH, OW, C), dtype=Y.dtype)
    for oh in range(OH):
        for ow in range(OW):
            win = Y[oh * stride: oh * stride + k, ow * stride: ow * stride + k, :]
            out[oh, ow, :] = win.reshape(-1, C).max(axis=0)
    return out
