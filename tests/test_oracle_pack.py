"""Pins for the oracle's bit-plane packing (O4): an independent unpack written here,
per-plane popcounts against per-bit column sums, the bit order and the zero padding."""
import numpy as np
import pytest

import oracle

U, TC, BP = oracle.UNSIGNED, oracle.TWOS_COMPLEMENT, oracle.BIPOLAR


def unpack(planes, depth, fmt):
    """Inverse of the packed format, written from its definition (test-side only)."""
    bits, rows, stride = planes.shape
    code = np.zeros((rows, depth), dtype=np.int64)
    for p in range(bits):
        for k in range(depth):
            bit = (planes[p, :, k // 64] >> np.uint64(k % 64)) & np.uint64(1)
            code[:, k] |= bit.astype(np.int64) << p
    if fmt == BP:
        return 2 * code - 1
    if fmt == TC:
        return np.where(code >= (1 << (bits - 1)), code - (1 << bits), code)
    return code


@pytest.mark.parametrize("depth", [1, 63, 64, 65, 128, 129, 300])
@pytest.mark.parametrize("bits,fmt", [(1, U), (2, U), (4, U), (1, TC), (2, TC), (3, TC), (4, TC), (1, BP)])
def test_roundtrip_and_padding(depth, bits, fmt):
    rng = np.random.default_rng(depth + bits)
    if fmt == BP:
        X = 2 * rng.integers(0, 2, size=(5, depth)) - 1
    elif fmt == TC:
        X = rng.integers(-(1 << (bits - 1)), 1 << (bits - 1), size=(5, depth))
    else:
        X = rng.integers(0, 1 << bits, size=(5, depth))
    P = oracle.pack(X, bits, fmt)
    assert P.dtype == np.uint64 and P.shape == (bits, 5, oracle.words_per_row(depth))
    assert np.array_equal(unpack(P, depth, fmt), X)
    # every bit at or beyond depth is zero
    full = np.unpackbits(P.view(np.uint8), axis=-1, bitorder="little")
    assert not full[:, :, depth:].any()
    # plane popcount = number of elements whose code has that bit set
    code = X & ((1 << bits) - 1) if fmt != BP else (X + 1) // 2
    for p in range(bits):
        assert full[p].sum() == ((code >> p) & 1).sum()


def test_bit_order_lsb_first():
    X = np.zeros((1, 130), dtype=np.int32)
    X[0, 0] = 1; X[0, 65] = 1; X[0, 129] = 2
    P = oracle.pack(X, 2, U)
    assert P.shape == (2, 1, 4)
    assert P[0, 0, 0] == 1 and P[0, 0, 1] == 2 and P[0, 0, 2] == 0
    assert P[1, 0, 2] == 2 and P[1, 0, 0] == 0


def test_words_per_row():
    assert [oracle.words_per_row(k) for k in (1, 64, 65, 128, 129, 2400, 9216)] == [2, 2, 2, 2, 4, 38, 144]
