"""Seeded synthetic inputs for the five benchmark configurations.

Input generation only: this module holds none of the method's arithmetic and is
the one module that both the tests of the CPU oracle and the GPU path draw their
inputs from.  The tensors take the shapes of the paper's AlexNet layers (Table 2)
and the value ranges of its W1A2 network (bipolar weights, unsigned 2-bit
activations, Sec. 4.2); they stand in for the trained HWGQ weights, which are
not available here.  Values are iid uniform over the stated range.

Every generator takes the config index and returns numpy arrays of *logical
values* (int8) and sorted int32 thresholds.
"""
from __future__ import annotations

import numpy as np
from scipy.stats import norm

BASE_SEED = 1709040600


def rng_for(cfg: int, stream: int = 0) -> np.random.Generator:
    return np.random.default_rng([BASE_SEED + cfg, stream])


def bipolar(rng, shape) -> np.ndarray:
    return (2 * rng.integers(0, 2, size=shape, dtype=np.int8) - 1).astype(np.int8)


def unsigned(rng, shape, bits: int) -> np.ndarray:
    return rng.integers(0, 1 << bits, size=shape, dtype=np.int8)


def twos_complement(rng, shape, bits: int) -> np.ndarray:
    return rng.integers(-(1 << (bits - 1)), 1 << (bits - 1), size=shape, dtype=np.int8)


def thresholds(rng, rows: int, obits: int, mu: float, sigma: float, jitter: int = 2) -> np.ndarray:
    """Per-row sorted int32 thresholds at the normal k/2^obits quantiles of
    N(mu, sigma^2) plus a small per-row integer jitter, so that outputs are close
    to uniform over 0..2^obits-1 when the accumulators are roughly normal."""
    T = (1 << obits) - 1
    q = norm.ppf(np.arange(1, T + 1) / (T + 1))
    base = np.rint(mu + sigma * q).astype(np.int64)
    thr = base[None, :] + rng.integers(-jitter, jitter + 1, size=(rows, T))
    thr.sort(axis=1)
    return thr.astype(np.int32)


def cfg1_tiny():
    """W1A2 tiny: W 64x256 bipolar, A 256x64 unsigned 2-bit."""
    r = rng_for(1)
    return dict(W=bipolar(r, (64, 256)), A=unsigned(r, (256, 64), 2))


def cfg2_square(size: int = 4096):
    """W2A2 square: W size^2 two's-complement 2-bit, A size^2 unsigned 2-bit."""
    r = rng_for(2)
    return dict(W=twos_complement(r, (size, size), 2), A=unsigned(r, (size, size), 2))


def cfg3_fc_chain(m6: int = 4096, k6: int = 9216, m7: int = 4096):
    """AlexNet fc6 -> fc7 at batch 1, W1A2, each followed by 3 thresholds per row.
    sigma = sqrt(E[a^2] K) with E[a^2] = 3.5 for uniform {0..3}; mean 0."""
    r = rng_for(3)
    return dict(
        W6=bipolar(r, (m6, k6)), x=unsigned(r, (k6, 1), 2),
        thr6=thresholds(r, m6, 2, 0.0, float(np.sqrt(3.5 * k6))),
        W7=bipolar(r, (m7, m6)),
        thr7=thresholds(r, m7, 2, 0.0, float(np.sqrt(3.5 * m6))))


def cfg4_conv2(H: int = 27, W: int = 27, C: int = 96, F: int = 256, k: int = 5, stride: int = 1, pad: int = 2):
    """AlexNet conv2 shape, W1A2: input HWC unsigned 2-bit, filters F x (k x k x C) bipolar."""
    r = rng_for(4)
    return dict(
        x=unsigned(r, (H, W, C), 2), filt=bipolar(r, (F, k, k, C)),
        thr=thresholds(r, F, 2, 0.0, float(np.sqrt(3.5 * k * k * C))),
        stride=stride, pad=pad)


def cfg5_w4a4(n: int, size: int = 8192):
    """W4A4: W size^2 two's-complement 4-bit, A size x n unsigned 4-bit, 15 thresholds
    per row around mu = E[w]E[a] K, sigma = sqrt(K (E[w^2]E[a^2] - (E[w]E[a])^2))."""
    r = rng_for(5)
    W = twos_complement(r, (size, size), 4)
    rn = rng_for(5, stream=n)
    mu = -0.5 * 7.5 * size
    sigma = float(np.sqrt((21.5 * 77.5 - (0.5 * 7.5) ** 2) * size))
    return dict(W=W, A=unsigned(rn, (size, n), 4), thr=thresholds(rn, size, 4, mu, sigma, jitter=8))


# The W1A2 layers of the paper's quantized AlexNet (Table 2), batch 1: name, kind, geometry.
# conv: (H, W, C, F, k, stride, pad); pool: (H, W, C, k, stride); fc: (M, K).
ALEXNET_INNER = [
    ("conv2", "conv", (27, 27, 96, 256, 5, 1, 2)),
    ("pool2", "pool", (27, 27, 256, 3, 2)),
    ("conv3", "conv", (13, 13, 256, 384, 3, 1, 1)),
    ("conv4", "conv", (13, 13, 384, 384, 3, 1, 1)),
    ("conv5", "conv", (13, 13, 384, 256, 3, 1, 1)),
    ("pool5", "pool", (13, 13, 256, 3, 2)),
    ("fc6", "fc", (4096, 9216)),
    ("fc7", "fc", (4096, 4096)),
]


def alexnet_inner(scale: int = 1):
    """Synthetic parameters for the chain conv2 .. fc7: bipolar weights, three sorted int32
    thresholds per output channel, and the 27 x 27 x 96 unsigned 2-bit input of conv2.
    `scale` > 1 divides the channel and row counts (smaller test instances); spatial sizes
    stay, so fc6's depth becomes 36 * (256 // scale)."""
    r = rng_for(6)
    layers = []
    x = None
    for name, kind, g in ALEXNET_INNER:
        if kind == "conv":
            H, W, C, F, k, s, p = g
            C, F = C // scale, F // scale
            if x is None:
                x = unsigned(r, (H, W, C), 2)
            K = k * k * C
            layers.append(dict(name=name, kind=kind, geom=(H, W, C, F, k, s, p), filt=bipolar(r, (F, k, k, C)),
                               thr=thresholds(r, F, 2, 0.0, float(np.sqrt(3.5 * K)))))
        elif kind == "pool":
            H, W, C, k, s = g
            layers.append(dict(name=name, kind=kind, geom=(H, W, C // scale, k, s)))
        else:
            M, K = g
            M = M // scale
            K = 36 * (256 // scale) if name == "fc6" else K // scale
            layers.append(dict(name=name, kind=kind, geom=(M, K), W=bipolar(r, (M, K)),
                               thr=thresholds(r, M, 2, 0.0, float(np.sqrt(3.5 * K)))))
    return x, layers
