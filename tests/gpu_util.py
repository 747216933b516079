"""Helpers for the GPU parity tests: move numpy arrays to the device and compare packed
planes / int32 results with the oracle's, element by element."""
import numpy as np
import torch

import oracle
import paper_1709_04060_amd as bs

FMT = {oracle.UNSIGNED: bs.BS_UNSIGNED, oracle.TWOS_COMPLEMENT: bs.BS_TWOS_COMPLEMENT, oracle.BIPOLAR: bs.BS_BIPOLAR}


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def planes_to_numpy(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


def planes_to_dev(p: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(p).view(np.int64)).cuda()


def draw(rng, shape, bits, fmt):
    if fmt == oracle.BIPOLAR:
        return (2 * rng.integers(0, 2, size=shape) - 1).astype(np.int8)
    if fmt == oracle.TWOS_COMPLEMENT:
        return rng.integers(-(1 << (bits - 1)), 1 << (bits - 1), size=shape).astype(np.int8)
    return rng.integers(0, 1 << bits, size=shape).astype(np.int8)


def assert_equal(got: np.ndarray, want: np.ndarray, what: str):
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        i = tuple(bad[0])
        raise AssertionError("%s: %d of %d elements differ; first at %s: got %s want %s"
                             % (what, len(bad), got.size, i, got[i], want[i]))


# ------------------------------------------------------------------ engines
ENGINE_NAMES = {bs.BS_ENGINE_AUTO: "auto", bs.BS_ENGINE_BITSERIAL: "bit-serial", bs.BS_ENGINE_DENSE_I8: "int8 matrix cores",
                bs.BS_ENGINE_DENSE_FP4: "fp4 matrix cores"}


def engines_for(wbits, wfmt, abits, afmt, K):
    """Every engine that can take a wbits x abits product of depth K from packed planes (bs format constants):
    the library's own choice, the AND-popcount kernels, the int8 matrix-core kernel, and the fp4 one for operands
    of at most two bits while its fp32 sum of products of unsigned codes is exact."""
    e = [bs.BS_ENGINE_AUTO, bs.BS_ENGINE_BITSERIAL]
    if K < (1 << 30):
        e.append(bs.BS_ENGINE_DENSE_I8)
        if wbits <= 2 and abits <= 2 and K * ((1 << wbits) - 1) * ((1 << abits) - 1) < (1 << 24):
            e.append(bs.BS_ENGINE_DENSE_FP4)
    return e


def gemm_all_engines(Wp, wfmt, Ap, afmt, K, what="gemm"):
    """bs_gemm on every engine that takes the case; the results must be identical.  Returns the int32 matrix
    (numpy), which the caller compares with the oracle."""
    first = None
    for eng in engines_for(Wp.shape[0], wfmt, Ap.shape[0], afmt, K):
        out = guarded_full((Wp.shape[1], Ap.shape[1]), -7, torch.int32)
        got = bs.bs_gemm(Wp, wfmt, Ap, afmt, K, out=out, engine=eng).cpu().numpy()
        check_guards()
        if first is None:
            first = got
        else:
            assert_equal(got, first, "%s: engine %s against engine auto" % (what, ENGINE_NAMES[eng]))
    return first


def gemm_threshold_all_engines(Wp, wfmt, Ap, afmt, K, thr, obits, what="gemm_threshold"):
    """bs_gemm_threshold on every engine, into buffers prefilled with ones and fenced by guard words; returns the
    packed planes (numpy uint64) after checking that all engines agree."""
    first = None
    M, N = Wp.shape[1], Ap.shape[1]
    for eng in engines_for(Wp.shape[0], wfmt, Ap.shape[0], afmt, K):
        out = guarded_full((obits, N, bs.bs_words_per_row(M)), -1, torch.int64)
        bs.bs_gemm_threshold(Wp, wfmt, Ap, afmt, K, thr, obits, out=out, engine=eng)
        got = planes_to_numpy(out)
        check_guards()
        if first is None:
            first = got
        else:
            assert_equal(got, first, "%s: engine %s against engine auto" % (what, ENGINE_NAMES[eng]))
    return first


def conv_threshold_all_engines(xp, afmt, B, H, W, C, Fp, wfmt, k, stride, pad, thr, obits, what="conv_threshold"):
    """bs_conv_threshold_batch on every engine that takes the layer (as a product F x Kl x B OH OW), into guarded
    buffers prefilled with ones; returns the packed planes (numpy uint64) after checking that all engines agree."""
    first = None
    F = Fp.shape[1]
    OH, OW = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    for eng in engines_for(Fp.shape[0], wfmt, xp.shape[0], afmt, bs.bs_lowered_depth(C, k, k)):
        out = guarded_full((obits, B * OH * OW, bs.bs_words_per_row(F)), -1, torch.int64)
        bs.bs_conv_threshold_batch(xp, afmt, B, H, W, C, Fp, wfmt, k, k, stride, pad, thr, obits, out=out, engine=eng)
        got = planes_to_numpy(out)
        check_guards()
        if first is None:
            first = got
        else:
            assert_equal(got, first, "%s: engine %s against engine auto" % (what, ENGINE_NAMES[eng]))
    return first


# ------------------------------------------------------------------ guard bands
# Every output buffer of a test sits inside a larger allocation with sentinel words before and behind it; a
# kernel that writes outside its output (a tile that ignores a ragged edge, a padding loop that runs too far)
# changes a sentinel and fails the test that ran it.
GUARD_BYTES = 4096          # on either side; a multiple of 256 so that the payload keeps the allocation's alignment
_SENTINEL = 0x5A
_live_guards = []


def guarded_empty(shape, dtype, device="cuda"):
    """A contiguous tensor of the given shape whose storage is fenced by GUARD_BYTES sentinel bytes on both sides."""
    shape = tuple(int(s) for s in shape)
    n = 1
    for s in shape:
        n *= s
    item = torch.empty((), dtype=dtype).element_size()
    payload = n * item
    pad = (-payload) % 256
    raw = torch.full((GUARD_BYTES + payload + pad + GUARD_BYTES,), _SENTINEL, dtype=torch.uint8, device=device)
    _live_guards.append((raw, payload))
    return raw[GUARD_BYTES:GUARD_BYTES + payload].view(dtype).reshape(shape)


def guarded_full(shape, fill, dtype, device="cuda"):
    t = guarded_empty(shape, dtype, device)
    t.fill_(fill)
    return t


def check_guards():
    """Synchronise and verify the sentinels of every guarded buffer handed out since the last check."""
    torch.cuda.synchronize()
    bad = []
    for raw, payload in _live_guards:
        front = raw[:GUARD_BYTES]
        back = raw[GUARD_BYTES + payload:]
        if not bool((front == _SENTINEL).all()) or not bool((back == _SENTINEL).all()):
            nf = int((front != _SENTINEL).sum())
            nb = int((back != _SENTINEL).sum())
            bad.append("payload of %d bytes: %d guard bytes changed before it, %d behind it" % (payload, nf, nb))
    _live_guards.clear()
    assert not bad, "out-of-bounds write: " + "; ".join(bad)


def install_guarded_allocator():
    """Route every output the binding allocates itself (out=None) through guarded_empty."""
    bs.set_output_allocator(lambda shape, dtype, device: guarded_empty(shape, dtype, device))
