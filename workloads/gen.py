"""Seeded tensor generators (numpy PCG64).  No method arithmetic lives here.

Every tensor t of layer l of configuration c is drawn from its own stream,
seed = BASE_SEED + 10000*c + 100*l + t, so any tensor can be regenerated alone.
Tensor ids t: 0 = input images, 1 = weights, 2 = thresholds, 3 = flips.
"""
import numpy as np

BASE_SEED = 230105126

T_INPUT, T_WEIGHT, T_THR, T_FLIP = 0, 1, 2, 3


def tensor_seed(config: int, layer: int, tensor: int) -> int:
    return BASE_SEED + 10000 * config + 100 * layer + tensor


def rng_for(config: int, layer: int, tensor: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(tensor_seed(config, layer, tensor)))


def draw_images(rng, n, h, w, c):
    """int8 NHWC images, integers uniform in [-127, 127] (stand-in for 8-bit pixels)."""
    return rng.integers(-127, 128, size=(n, h, w, c), dtype=np.int8)


def draw_pm1(rng, shape):
    """+1/-1 values, Bernoulli(1/2), as int8."""
    bits = rng.integers(0, 2, size=shape, dtype=np.int8)
    return (2 * bits - 1).astype(np.int8)


def draw_bits_pm1(rng, rows, k):
    """Random +-1 matrix [rows][k] for the GEMM sweep, drawn in row blocks to bound memory."""
    out = np.empty((rows, k), dtype=np.int8)
    step = max(1, (1 << 24) // max(k, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        b = rng.integers(0, 2, size=(r1 - r0, k), dtype=np.int8)
        np.multiply(b, 2, out=b)
        np.subtract(b, 1, out=b)
        out[r0:r1] = b
    return out


def draw_threshold(rng, channels, fan_in):
    """Per-channel int32 thresholds, integers uniform in [-floor(K/8), floor(K/8)]."""
    b = fan_in // 8
    return rng.integers(-b, b + 1, size=(channels,), dtype=np.int32)


def draw_flip(rng, channels):
    """Per-channel comparison-direction flags, Bernoulli(1/2), uint8 in {0,1}."""
    return rng.integers(0, 2, size=(channels,), dtype=np.uint8)
