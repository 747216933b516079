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
