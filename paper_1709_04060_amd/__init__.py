"""Thin Python binding of libbsgemm (C ABI in include/bsgemm.h).

Argument marshalling only: every step of the path runs in the HIP kernels of the
library.  PyTorch is used for device memory and streams, nothing else.  There is no
CPU fallback: if the library is missing or a call fails, an exception is raised.

Functions carry the names of the C entry points.  Tensors must live on the GPU; the
functions enqueue on torch's current stream and return without synchronising.
"""
from __future__ import annotations

import ctypes
import os

import torch  # imported before the library so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
# BSGEMM_LIBRARY names another build of the library (an instrumented one, say); the default is the in-tree build
LIB_PATH = os.environ.get("BSGEMM_LIBRARY") or os.path.join(_HERE, "libbsgemm.so")

BS_OK = 0
BS_ERR_INVALID_ARG, BS_ERR_UNSUPPORTED, BS_ERR_ALIGNMENT, BS_ERR_OVERFLOW_RISK, BS_ERR_LAUNCH = -1, -2, -3, -4, -5
BS_UNSIGNED, BS_TWOS_COMPLEMENT, BS_BIPOLAR = 0, 1, 2
BS_I8, BS_I32 = 0, 1
# engines: bs_choose_engine returns one of the first three; BS_ENGINE_AUTO (bs_gemm_on and friends) lets the library choose
BS_ENGINE_BITSERIAL, BS_ENGINE_DENSE_I8, BS_ENGINE_DENSE_FP4, BS_ENGINE_AUTO = 0, 1, 2, 3

EXPORTS = ("bs_words_per_row", "bs_lowered_depth", "bs_pack_planes", "bs_gemm", "bs_gemm_topbits", "bs_threshold_activate",
           "bs_gemm_threshold", "bs_gemm_on", "bs_gemm_threshold_on", "bs_im2col_interleaved", "bs_im2col_interleaved_batch", "bs_conv_threshold", "bs_conv_threshold_batch", "bs_conv_threshold_batch_on", "bs_pool_conv_threshold_batch", "bs_maxpool_packed",
           "bs_maxpool_packed_batch",
           "bs_unpack_planes", "bs_gemm_i8", "bs_gemm_i8_threshold", "bs_unpack_planes_fp4", "bs_gemm_fp4",
           "bs_gemm_fp4_threshold", "bs_streamline_collapse",
           "bs_streamline_thresholds", "bs_choose_engine", "bs_planes_tile", "bs_probe_popcount_rate", "bs_probe_stream_read", "bs_status_string", "bs_version")


class BsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, status_string(status), status))


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libbsgemm.so (built in-tree by paper_1709_04060_amd.build).  Fails loudly."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libbsgemm.so is not built: run `python -m paper_1709_04060_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
    lib.bs_words_per_row.argtypes = [i64]; lib.bs_words_per_row.restype = i64
    lib.bs_lowered_depth.argtypes = [i64, i64, i64]; lib.bs_lowered_depth.restype = i64
    lib.bs_pack_planes.argtypes = [vp, i32, i64, i64, i64, i32, i32, i32, vp, vp]; lib.bs_pack_planes.restype = i32
    lib.bs_gemm.argtypes = [vp, i32, i32, vp, i32, i32, i64, i64, i64, vp, i64, vp]; lib.bs_gemm.restype = i32
    lib.bs_gemm_topbits.argtypes = [vp, i32, i32, vp, i32, i32, i64, i64, i64, i32, vp, i64, vp]; lib.bs_gemm_topbits.restype = i32
    lib.bs_threshold_activate.argtypes = [vp, i64, i64, i64, vp, i32, vp, vp]; lib.bs_threshold_activate.restype = i32
    lib.bs_gemm_threshold.argtypes = [vp, i32, i32, vp, i32, i32, i64, i64, i64, vp, i32, vp, vp]
    lib.bs_gemm_threshold.restype = i32
    lib.bs_gemm_on.argtypes = [i32] + lib.bs_gemm.argtypes; lib.bs_gemm_on.restype = i32
    lib.bs_gemm_threshold_on.argtypes = [i32] + lib.bs_gemm_threshold.argtypes; lib.bs_gemm_threshold_on.restype = i32
    lib.bs_im2col_interleaved.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.bs_im2col_interleaved.restype = i32
    lib.bs_conv_threshold.argtypes = [vp, i32, i32, i32, i32, i32, vp, i32, i32, i32, i32, i32, i32, i32, vp, i32, vp, vp]
    lib.bs_conv_threshold.restype = i32
    lib.bs_im2col_interleaved_batch.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.bs_im2col_interleaved_batch.restype = i32
    lib.bs_conv_threshold_batch.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, i32, i32, i32, i32, i32, i32, i32, vp, i32,
                                            vp, vp]
    lib.bs_conv_threshold_batch.restype = i32
    lib.bs_conv_threshold_batch_on.argtypes = [i32] + lib.bs_conv_threshold_batch.argtypes
    lib.bs_conv_threshold_batch_on.restype = i32
    # in, abits, B, H, W, C, pool_k, pool_stride, Fp, wbits, wfmt, F, kh, kw, stride, pad, thr, obits, Yp, stream
    lib.bs_pool_conv_threshold_batch.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, vp, i32, i32, i32, i32, i32, i32, i32,
                                                 vp, i32, vp, vp]
    lib.bs_pool_conv_threshold_batch.restype = i32
    lib.bs_maxpool_packed_batch.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.bs_maxpool_packed_batch.restype = i32
    lib.bs_maxpool_packed.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp]; lib.bs_maxpool_packed.restype = i32
    lib.bs_unpack_planes.argtypes = [vp, i32, i32, i64, i64, vp, i64, vp]; lib.bs_unpack_planes.restype = i32
    lib.bs_gemm_i8.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, i64, vp]; lib.bs_gemm_i8.restype = i32
    lib.bs_gemm_i8_threshold.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, i32, vp, vp]
    lib.bs_gemm_i8_threshold.restype = i32
    f64 = ctypes.c_double
    lib.bs_unpack_planes_fp4.argtypes = [vp, i32, i32, i64, i64, vp, i64, vp]; lib.bs_unpack_planes_fp4.restype = i32
    lib.bs_gemm_fp4.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, i64, vp]; lib.bs_gemm_fp4.restype = i32
    lib.bs_gemm_fp4_threshold.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, i32, vp, vp]
    lib.bs_gemm_fp4_threshold.restype = i32
    lib.bs_streamline_collapse.argtypes = [i64, f64, f64, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.bs_streamline_collapse.restype = i32
    lib.bs_streamline_thresholds.argtypes = [vp, i32, vp, vp, i64, vp, vp]; lib.bs_streamline_thresholds.restype = i32
    lib.bs_choose_engine.argtypes = [i32, i32, i32, i32, i64, i64, i64]; lib.bs_choose_engine.restype = i32
    lib.bs_planes_tile.argtypes = [i64, i64, vp, vp]; lib.bs_planes_tile.restype = i32
    lib.bs_probe_popcount_rate.argtypes = [vp, i32, i32, vp]; lib.bs_probe_popcount_rate.restype = i32
    lib.bs_probe_stream_read.argtypes = [vp, i64, vp, i32, i32, vp]; lib.bs_probe_stream_read.restype = i32
    lib.bs_status_string.argtypes = [i32]; lib.bs_status_string.restype = ctypes.c_char_p
    lib.bs_version.argtypes = []; lib.bs_version.restype = i32
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().bs_status_string(int(status)).decode()


def bs_version() -> int:
    return int(load_library().bs_version())


def bs_words_per_row(depth: int) -> int:
    return int(load_library().bs_words_per_row(int(depth)))


def bs_lowered_depth(C: int, kh: int, kw: int) -> int:
    return int(load_library().bs_lowered_depth(int(C), int(kh), int(kw)))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(st: int, where: str):
    if st != BS_OK:
        raise BsError(st, where)


def _dev(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda:
        raise ValueError("%s must be a GPU tensor" % name)
    return t.data_ptr()


# Output buffers the binding allocates itself (out=None) come from this function; a caller
# with an allocator of their own (a memory pool, buffers with guard bands) can replace it.
def _default_new_output(shape, dtype, device) -> torch.Tensor:
    return torch.empty(tuple(shape), dtype=dtype, device=device)


_new_output = _default_new_output


def set_output_allocator(fn=None) -> None:
    """fn(shape, dtype, device) -> contiguous GPU tensor; None restores torch.empty."""
    global _new_output
    _new_output = fn or _default_new_output


def _planes(bits: int, rows: int, depth: int, device) -> torch.Tensor:
    # uint64 planes are carried as int64 tensors (same bytes)
    return _new_output((bits, rows, bs_words_per_row(depth)), torch.int64, device)


# ---- argument validation (host only).  The library trusts sizes: a depth larger than the
# buffers really hold would make a kernel read past them, and a wrong dtype or a strided view
# would give wrong numbers with BS_OK.  Every wrapper therefore checks dtype, contiguity and
# shape against the sizes it hands over, and raises ValueError before anything is called.
def _want_planes(t: torch.Tensor, name: str, depth: int, bits: int | None = None, rows: int | None = None) -> None:
    if t.dtype != torch.int64:
        raise ValueError("%s must be int64 (uint64 bit planes), got %s" % (name, t.dtype))
    if t.dim() != 3:
        raise ValueError("%s must be 3-D [bits][rows][words], got %d-D" % (name, t.dim()))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if not 1 <= t.shape[0] <= 4:
        raise ValueError("%s: 1..4 bit planes expected, got %d" % (name, t.shape[0]))
    if bits is not None and t.shape[0] != bits:
        raise ValueError("%s must hold %d planes, got %d" % (name, bits, t.shape[0]))
    if rows is not None and t.shape[1] != rows:
        raise ValueError("%s must hold %d rows, got %d" % (name, rows, t.shape[1]))
    if depth <= 0 or t.shape[2] != bs_words_per_row(depth):
        raise ValueError("%s: rows of %d words do not match depth %d (bs_words_per_row = %d)"
                         % (name, t.shape[2], depth, bs_words_per_row(depth)))


def _want_thr(thr: torch.Tensor, M: int, obits: int) -> None:
    if not 1 <= obits <= 4:
        raise ValueError("obits must be 1..4, got %d" % obits)
    if thr.dtype != torch.int32:
        raise ValueError("thr must be int32, got %s" % thr.dtype)
    if thr.dim() != 2 or tuple(thr.shape) != (M, (1 << obits) - 1):
        raise ValueError("thr must have shape [%d][%d], got %s" % (M, (1 << obits) - 1, tuple(thr.shape)))
    if not thr.is_contiguous():
        raise ValueError("thr must be contiguous")


def _want_c(C: torch.Tensor, M: int, N: int, name: str = "out") -> None:
    if C.dtype != torch.int32:
        raise ValueError("%s must be int32, got %s" % (name, C.dtype))
    if C.dim() != 2 or tuple(C.shape) != (M, N):
        raise ValueError("%s must have shape [%d][%d], got %s" % (name, M, N, tuple(C.shape)))
    if C.stride(1) != 1 or (M > 1 and C.stride(0) < N):
        raise ValueError("%s must have unit column stride and a row stride >= %d" % (name, N))


def _want_dense(t: torch.Tensor, name: str, kbytes: int, dtype) -> None:
    if t.dtype != dtype:
        raise ValueError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("%s must be 2-D with depth-contiguous rows" % name)
    if kbytes <= 0 or t.shape[1] < kbytes or (t.shape[0] > 1 and t.stride(0) < kbytes):
        raise ValueError("%s: rows of %d bytes (stride %d) are shorter than the depth's %d bytes"
                         % (name, t.shape[1], t.stride(0), kbytes))


def _conv_geometry(x: torch.Tensor, B: int, H: int, W: int, C: int, Fp: torch.Tensor, kh: int, kw: int,
                   stride: int, pad: int):
    if min(B, H, W, C, kh, kw, stride) <= 0 or pad < 0 or H + 2 * pad < kh or W + 2 * pad < kw:
        raise ValueError("bad convolution geometry")
    _want_planes(x, "x", C, rows=B * H * W)
    _want_planes(Fp, "Fp", bs_lowered_depth(C, kh, kw))
    return (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1


def bs_pack_planes(src: torch.Tensor, bits: int, fmt: int, depth_is_strided: bool = False,
                   out: torch.Tensor | None = None) -> torch.Tensor:
    """Pack a 2-D int8/int32 matrix of logical values into bit planes [bits][rows][S].
    depth_is_strided=False: src is [rows][depth]; True: src is [depth][rows]."""
    if src.dim() != 2 or src.stride(1) != 1:
        raise ValueError("src must be 2-D with a contiguous last dimension")
    if src.dtype not in (torch.int8, torch.int32):
        raise ValueError("src must be int8 or int32, got %s" % src.dtype)
    dtype = {torch.int8: BS_I8, torch.int32: BS_I32}[src.dtype]
    rows, depth = (src.shape[1], src.shape[0]) if depth_is_strided else (src.shape[0], src.shape[1])
    if src.shape[0] > 1 and src.stride(0) < src.shape[1]:
        raise ValueError("src rows overlap (row stride below the row length)")
    # a single row has no meaningful row stride (frameworks report anything): pass the row length
    ld = src.stride(0) if src.shape[0] > 1 else src.shape[1]
    if out is None:
        out = _planes(bits, rows, depth, src.device)
    _want_planes(out, "out", depth, bits=bits, rows=rows)
    st = load_library().bs_pack_planes(_dev(src, "src"), dtype, rows, depth, ld, int(bool(depth_is_strided)),
                                       bits, fmt, _dev(out, "out"), _stream())
    _check(st, "bs_pack_planes")
    return out


def _gemm_operands(Wp: torch.Tensor, Ap: torch.Tensor, K: int):
    _want_planes(Wp, "Wp", K)
    _want_planes(Ap, "Ap", K)
    return Wp.shape[0], Wp.shape[1], Ap.shape[0], Ap.shape[1]


def bs_gemm(Wp: torch.Tensor, wfmt: int, Ap: torch.Tensor, afmt: int, K: int,
            out: torch.Tensor | None = None, engine: int = BS_ENGINE_AUTO) -> torch.Tensor:
    """C[M][N] (int32) = W . A from packed planes Wp [w][M][S], Ap [a][N][S].  engine: BS_ENGINE_AUTO lets
    the library take the fastest engine (bs_gemm); any other value asks for that engine (bs_gemm_on)."""
    wbits, M, abits, N = _gemm_operands(Wp, Ap, K)
    if out is None:
        out = _new_output((M, N), torch.int32, Wp.device)
    _want_c(out, M, N)
    lib = load_library()
    if engine == BS_ENGINE_AUTO:
        st = lib.bs_gemm(_dev(Wp, "Wp"), wbits, wfmt, _dev(Ap, "Ap"), abits, afmt, M, N, K,
                         _dev(out, "out"), out.stride(0), _stream())
    else:
        st = lib.bs_gemm_on(int(engine), _dev(Wp, "Wp"), wbits, wfmt, _dev(Ap, "Ap"), abits, afmt, M, N, K,
                            _dev(out, "out"), out.stride(0), _stream())
    _check(st, "bs_gemm")
    return out


def bs_threshold_activate(C: torch.Tensor, thr: torch.Tensor, obits: int,
                          out: torch.Tensor | None = None) -> torch.Tensor:
    """Yp [obits][N][S_M]: bit planes of the number of thresholds thr[m][:] that C[m][n] reaches."""
    if C.dim() != 2:
        raise ValueError("C must be 2-D")
    M, N = C.shape
    _want_c(C, M, N, "C")
    _want_thr(thr, M, obits)
    if out is None:
        out = _planes(obits, N, M, C.device)
    _want_planes(out, "out", M, bits=obits, rows=N)
    st = load_library().bs_threshold_activate(_dev(C, "C"), C.stride(0), M, N, _dev(thr, "thr"), obits,
                                              _dev(out, "out"), _stream())
    _check(st, "bs_threshold_activate")
    return out


def bs_gemm_threshold(Wp: torch.Tensor, wfmt: int, Ap: torch.Tensor, afmt: int, K: int, thr: torch.Tensor,
                      obits: int, out: torch.Tensor | None = None, engine: int = BS_ENGINE_AUTO) -> torch.Tensor:
    """Fused bs_gemm + bs_threshold_activate; the int32 product never leaves the chip.  engine as in bs_gemm."""
    wbits, M, abits, N = _gemm_operands(Wp, Ap, K)
    _want_thr(thr, M, obits)
    if out is None:
        out = _planes(obits, N, M, Wp.device)
    _want_planes(out, "out", M, bits=obits, rows=N)
    lib = load_library()
    if engine == BS_ENGINE_AUTO:
        st = lib.bs_gemm_threshold(_dev(Wp, "Wp"), wbits, wfmt, _dev(Ap, "Ap"), abits, afmt, M, N, K,
                                   _dev(thr, "thr"), obits, _dev(out, "out"), _stream())
    else:
        st = lib.bs_gemm_threshold_on(int(engine), _dev(Wp, "Wp"), wbits, wfmt, _dev(Ap, "Ap"), abits, afmt, M, N, K,
                                      _dev(thr, "thr"), obits, _dev(out, "out"), _stream())
    _check(st, "bs_gemm_threshold")
    return out


def bs_im2col_interleaved(x: torch.Tensor, H: int, W: int, C: int, kh: int, kw: int, stride: int, pad: int,
                          out: torch.Tensor | None = None) -> torch.Tensor:
    """Lower packed HWC planes x [abits][H*W][S_C] to packed columns [abits][OH*OW][S_Kl]."""
    return bs_im2col_interleaved_batch(x, 1, H, W, C, kh, kw, stride, pad, out=out)


def bs_im2col_interleaved_batch(x: torch.Tensor, B: int, H: int, W: int, C: int, kh: int, kw: int, stride: int, pad: int,
                                out: torch.Tensor | None = None) -> torch.Tensor:
    """Lower B packed HWC maps x [abits][B*H*W][S_C] to packed columns [abits][B*OH*OW][S_Kl]."""
    if min(B, H, W, C, kh, kw, stride) <= 0 or pad < 0 or H + 2 * pad < kh or W + 2 * pad < kw:
        raise ValueError("bad convolution geometry")
    _want_planes(x, "x", C, rows=B * H * W)
    abits = x.shape[0]
    OH = (H + 2 * pad - kh) // stride + 1
    OW = (W + 2 * pad - kw) // stride + 1
    Kl = bs_lowered_depth(C, kh, kw)
    if out is None:
        out = _planes(abits, B * OH * OW, Kl, x.device)
    _want_planes(out, "out", Kl, bits=abits, rows=B * OH * OW)
    st = load_library().bs_im2col_interleaved_batch(_dev(x, "x"), abits, B, H, W, C, kh, kw, stride, pad,
                                                    _dev(out, "out"), _stream())
    _check(st, "bs_im2col_interleaved_batch")
    return out


def bs_conv_threshold(x: torch.Tensor, afmt: int, H: int, W: int, C: int, Fp: torch.Tensor, wfmt: int,
                      kh: int, kw: int, stride: int, pad: int, thr: torch.Tensor, obits: int,
                      out: torch.Tensor | None = None, engine: int = BS_ENGINE_AUTO) -> torch.Tensor:
    """Convolution + thresholding on packed HWC planes x [abits][H*W][S_C] with filter planes
    Fp [wbits][F][S_Kl]; returns the packed HWC planes [obits][OH*OW][S_F] of the output map."""
    return bs_conv_threshold_batch(x, afmt, 1, H, W, C, Fp, wfmt, kh, kw, stride, pad, thr, obits, out=out, engine=engine)


def bs_conv_threshold_batch(x: torch.Tensor, afmt: int, B: int, H: int, W: int, C: int, Fp: torch.Tensor, wfmt: int,
                            kh: int, kw: int, stride: int, pad: int, thr: torch.Tensor, obits: int,
                            out: torch.Tensor | None = None, engine: int = BS_ENGINE_AUTO) -> torch.Tensor:
    """bs_conv_threshold for B images: x [abits][B*H*W][S_C] -> [obits][B*OH*OW][S_F].  engine as in bs_gemm."""
    OH, OW = _conv_geometry(x, B, H, W, C, Fp, kh, kw, stride, pad)
    abits = x.shape[0]
    wbits, F, _ = Fp.shape
    _want_thr(thr, F, obits)
    if out is None:
        out = _planes(obits, B * OH * OW, F, x.device)
    _want_planes(out, "out", F, bits=obits, rows=B * OH * OW)
    st = load_library().bs_conv_threshold_batch_on(int(engine), _dev(x, "x"), abits, afmt, B, H, W, C, _dev(Fp, "Fp"), wbits,
                                                   wfmt, F, kh, kw, stride, pad, _dev(thr, "thr"), obits, _dev(out, "out"),
                                                   _stream())
    _check(st, "bs_conv_threshold_batch")
    return out


def bs_pool_conv_threshold_batch(x: torch.Tensor, B: int, H: int, W: int, C: int, pool_k: int, pool_stride: int,
                                 Fp: torch.Tensor, wfmt: int, kh: int, kw: int, stride: int, pad: int,
                                 thr: torch.Tensor, obits: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """bs_maxpool_packed_batch + bs_conv_threshold_batch in one call: x [abits][B*H*W][S_C] is the unpooled map
    (unsigned codes); the convolution reads its pool_k x pool_k / pool_stride maximum."""
    if min(B, H, W, C, pool_k, pool_stride) <= 0 or pool_k > H or pool_k > W:
        raise ValueError("bad pooling geometry")
    PH, PW = (H - pool_k) // pool_stride + 1, (W - pool_k) // pool_stride + 1
    if min(kh, kw, stride) <= 0 or pad < 0 or PH + 2 * pad < kh or PW + 2 * pad < kw:
        raise ValueError("bad convolution geometry")
    _want_planes(x, "x", C, rows=B * H * W)
    _want_planes(Fp, "Fp", bs_lowered_depth(C, kh, kw))
    OH, OW = (PH + 2 * pad - kh) // stride + 1, (PW + 2 * pad - kw) // stride + 1
    abits = x.shape[0]
    wbits, F, _ = Fp.shape
    _want_thr(thr, F, obits)
    if out is None:
        out = _planes(obits, B * OH * OW, F, x.device)
    _want_planes(out, "out", F, bits=obits, rows=B * OH * OW)
    st = load_library().bs_pool_conv_threshold_batch(_dev(x, "x"), abits, B, H, W, C, pool_k, pool_stride, _dev(Fp, "Fp"),
                                                     wbits, wfmt, F, kh, kw, stride, pad, _dev(thr, "thr"), obits,
                                                     _dev(out, "out"), _stream())
    _check(st, "bs_pool_conv_threshold_batch")
    return out


def bs_maxpool_packed_batch(x: torch.Tensor, B: int, H: int, W: int, C: int, k: int, stride: int,
                            out: torch.Tensor | None = None) -> torch.Tensor:
    """Max pooling of B packed HWC maps x [bits][B*H*W][S_C] -> [bits][B*OH*OW][S_C]."""
    if min(B, H, W, C, k, stride) <= 0 or k > H or k > W:
        raise ValueError("bad pooling geometry")
    _want_planes(x, "x", C, rows=B * H * W)
    bits = x.shape[0]
    OH, OW = (H - k) // stride + 1, (W - k) // stride + 1
    if out is None:
        out = _planes(bits, B * OH * OW, C, x.device)
    _want_planes(out, "out", C, bits=bits, rows=B * OH * OW)
    st = load_library().bs_maxpool_packed_batch(_dev(x, "x"), bits, B, H, W, C, k, stride, _dev(out, "out"), _stream())
    _check(st, "bs_maxpool_packed_batch")
    return out


def bs_maxpool_packed(x: torch.Tensor, H: int, W: int, C: int, k: int, stride: int,
                      out: torch.Tensor | None = None) -> torch.Tensor:
    """Max pooling of packed HWC planes x [bits][H*W][S_C] -> [bits][OH*OW][S_C]."""
    return bs_maxpool_packed_batch(x, 1, H, W, C, k, stride, out=out)


def bs_unpack_planes(planes: torch.Tensor, fmt: int, depth: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """planes [bits][rows][S] -> int8 [rows][ld] of logical values (ld = depth rounded up to 16)."""
    _want_planes(planes, "planes", depth)
    bits, rows, _ = planes.shape
    ld = 16 * ((depth + 15) // 16)
    if out is None:
        out = _new_output((rows, ld), torch.int8, planes.device)
    _want_dense(out, "out", ld, torch.int8)
    if out.shape[0] != rows:
        raise ValueError("out must hold %d rows, got %d" % (rows, out.shape[0]))
    st = load_library().bs_unpack_planes(_dev(planes, "planes"), bits, fmt, rows, depth, _dev(out, "out"),
                                         out.stride(0), _stream())
    _check(st, "bs_unpack_planes")
    return out


def _dense_call(fn_name: str, W: torch.Tensor, At: torch.Tensor, K: int, kbytes: int, dtype, thr, obits, out):
    _want_dense(W, "W", kbytes, dtype)
    _want_dense(At, "At", kbytes, dtype)
    M, N = W.shape[0], At.shape[0]
    lib = load_library()
    if thr is None:
        if out is None:
            out = _new_output((M, N), torch.int32, W.device)
        _want_c(out, M, N)
        st = getattr(lib, fn_name)(_dev(W, "W"), W.stride(0), _dev(At, "At"), At.stride(0), M, N, K,
                                   _dev(out, "out"), out.stride(0), _stream())
    else:
        _want_thr(thr, M, obits)
        if out is None:
            out = _planes(obits, N, M, W.device)
        _want_planes(out, "out", M, bits=obits, rows=N)
        st = getattr(lib, fn_name)(_dev(W, "W"), W.stride(0), _dev(At, "At"), At.stride(0), M, N, K,
                                   _dev(thr, "thr"), obits, _dev(out, "out"), _stream())
    _check(st, fn_name)
    return out


def bs_gemm_i8(W: torch.Tensor, At: torch.Tensor, K: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """Dense engine: C[M][N] (int32) from int8 W [M][>=K] and At [N][>=K] (depth-contiguous rows)."""
    return _dense_call("bs_gemm_i8", W, At, K, K, torch.int8, None, 0, out)


def bs_gemm_i8_threshold(W: torch.Tensor, At: torch.Tensor, K: int, thr: torch.Tensor, obits: int,
                         out: torch.Tensor | None = None) -> torch.Tensor:
    """Dense engine with the fused thresholding epilogue; output planes as bs_gemm_threshold."""
    return _dense_call("bs_gemm_i8_threshold", W, At, K, K, torch.int8, thr, obits, out)


def bs_choose_engine(wbits: int, wfmt: int, abits: int, afmt: int, M: int, N: int, K: int) -> int:
    """Host-only: the engine (BS_ENGINE_*) expected to be fastest for a wbits x abits product of shape M x K x N."""
    return load_library().bs_choose_engine(wbits, wfmt, abits, afmt, M, N, K)


def bs_planes_tile(M: int, N: int) -> tuple[int, int, int]:
    """Host-only: (tile edge 256 or 128, rounds over the chip, tiles) of the matrix-core kernel on packed planes for
    an M x N output."""
    rounds, tiles = ctypes.c_longlong(0), ctypes.c_longlong(0)
    tile = load_library().bs_planes_tile(int(M), int(N), ctypes.byref(rounds), ctypes.byref(tiles))
    return int(tile), int(rounds.value), int(tiles.value)


def bs_probe_popcount_rate(sink: torch.Tensor, passes: int) -> int:
    """Launch the AND + popcount rate probe with one workgroup per element of sink (int32, device);
    returns the lane-operations of the launch (the caller times it)."""
    if sink.dtype != torch.int32 or not sink.is_contiguous():
        raise ValueError("sink must be a contiguous int32 tensor")
    wgs = sink.numel()
    st = load_library().bs_probe_popcount_rate(_dev(sink, "sink"), wgs, passes, _stream())
    _check(st, "bs_probe_popcount_rate")
    return wgs * 256 * passes * 32


def bs_probe_stream_read(src: torch.Tensor, sink: torch.Tensor, non_temporal: bool = False) -> int:
    """Launch the streaming-read probe over the bytes of src (contiguous, a multiple of 16 bytes) with one
    workgroup per element of sink (int32, device); returns the bytes read (the caller times it)."""
    if not src.is_contiguous() or (src.numel() * src.element_size()) % 16:
        raise ValueError("src must be contiguous and a multiple of 16 bytes long")
    if sink.dtype != torch.int32 or not sink.is_contiguous():
        raise ValueError("sink must be a contiguous int32 tensor")
    nbytes = src.numel() * src.element_size()
    st = load_library().bs_probe_stream_read(_dev(src, "src"), nbytes, _dev(sink, "sink"), sink.numel(),
                                             int(bool(non_temporal)), _stream())
    _check(st, "bs_probe_stream_read")
    return nbytes


def bs_unpack_planes_fp4(planes: torch.Tensor, fmt: int, depth: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """planes [bits][rows][S] -> uint8 [rows][ld] of E2M1 codes, two per byte (ld = 16 * ceil(depth / 32))."""
    _want_planes(planes, "planes", depth)
    bits, rows, _ = planes.shape
    ld = 16 * ((depth + 31) // 32)
    if out is None:
        out = _new_output((rows, ld), torch.uint8, planes.device)
    _want_dense(out, "out", ld, torch.uint8)
    if out.shape[0] != rows:
        raise ValueError("out must hold %d rows, got %d" % (rows, out.shape[0]))
    st = load_library().bs_unpack_planes_fp4(_dev(planes, "planes"), bits, fmt, rows, depth, _dev(out, "out"),
                                             out.stride(0), _stream())
    _check(st, "bs_unpack_planes_fp4")
    return out


def bs_gemm_fp4(W: torch.Tensor, At: torch.Tensor, K: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """Dense fp4 engine: C[M][N] (int32) from E2M1-coded W [M][>= K/2 bytes] and At [N][>= K/2 bytes]."""
    return _dense_call("bs_gemm_fp4", W, At, K, (K + 1) // 2, torch.uint8, None, 0, out)


def bs_gemm_fp4_threshold(W: torch.Tensor, At: torch.Tensor, K: int, thr: torch.Tensor, obits: int,
                          out: torch.Tensor | None = None) -> torch.Tensor:
    """Dense fp4 engine with the fused thresholding epilogue; output planes as bs_gemm_threshold."""
    return _dense_call("bs_gemm_fp4_threshold", W, At, K, (K + 1) // 2, torch.uint8, thr, obits, out)


def _np_ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def bs_streamline_collapse(M: int, a_q: float = 1.0, b_q: float = 0.0, rowsum_w=None, alpha=None, gamma=None,
                           beta=None, mu=None, sigma=None):
    """Host-side: per-channel (a, b) of y = a x + b from the layer's float pieces (numpy arrays)."""
    import numpy as np
    f = lambda v: None if v is None else np.ascontiguousarray(v, dtype=np.float64)
    rs = None if rowsum_w is None else np.ascontiguousarray(rowsum_w, dtype=np.int64)
    alpha, gamma, beta, mu, sigma = f(alpha), f(gamma), f(beta), f(mu), f(sigma)
    for v in (rs, alpha, gamma, beta, mu, sigma):
        if v is not None and v.shape != (M,):
            raise ValueError("per-channel arrays must have shape (%d,)" % M)
    a, b = np.empty(M, dtype=np.float64), np.empty(M, dtype=np.float64)
    st = load_library().bs_streamline_collapse(M, float(a_q), float(b_q), _np_ptr(rs), _np_ptr(alpha), _np_ptr(gamma),
                                               _np_ptr(beta), _np_ptr(mu), _np_ptr(sigma), _np_ptr(a), _np_ptr(b))
    _check(st, "bs_streamline_collapse")
    return a, b


def bs_streamline_thresholds(t, a, b):
    """Host-side: integer thresholds thr [M][T] and the per-channel negate flags (numpy arrays)."""
    import numpy as np
    t = np.ascontiguousarray(t, dtype=np.float64)
    a = np.ascontiguousarray(a, dtype=np.float64)
    b = np.ascontiguousarray(b, dtype=np.float64)
    if t.ndim != 1 or a.ndim != 1 or a.shape != b.shape:
        raise ValueError("t [T], a [M], b [M] expected")
    M, T = a.shape[0], t.shape[0]
    thr = np.empty((M, T), dtype=np.int32)
    neg = np.empty(M, dtype=np.uint8)
    st = load_library().bs_streamline_thresholds(_np_ptr(t), T, _np_ptr(a), _np_ptr(b), M, _np_ptr(thr), _np_ptr(neg))
    _check(st, "bs_streamline_thresholds")
    return thr, neg


def bs_gemm_topbits(Wp: torch.Tensor, wfmt: int, Ap: torch.Tensor, afmt: int, K: int, min_shift: int,
                    out: torch.Tensor | None = None) -> torch.Tensor:
    """Approximate C from the plane pairs with i + j >= min_shift only."""
    wbits, M, abits, N = _gemm_operands(Wp, Ap, K)
    if out is None:
        out = _new_output((M, N), torch.int32, Wp.device)
    _want_c(out, M, N)
    st = load_library().bs_gemm_topbits(_dev(Wp, "Wp"), wbits, wfmt, _dev(Ap, "Ap"), abits, afmt, M, N, K, min_shift,
                                        _dev(out, "out"), out.stride(0), _stream())
    _check(st, "bs_gemm_topbits")
    return out
