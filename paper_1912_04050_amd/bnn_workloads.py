"""Seeded synthetic inputs for the binary convolution layer.

This module only *constructs inputs* (random +1 / -1 tensors, thresholds, batch-norm
parameters, layer shapes); it holds none of the layer's arithmetic.  Both the CPU oracle's
tests and the HIP path's tests feed from it so that they see identical data.  Random numbers
come from the counter-based splitmix64 streams of ``workloads.py``.

No dataset or trained model is involved: weights and activations are fair coin flips, which is
what a xor / popcount kernel's running time depends on (nothing: it is data-independent) and
what its correctness tests need (every bit pattern equally likely).
"""
from __future__ import annotations

import numpy as np

from .workloads import DEFAULT_SEED, stream, uniform_double, uniform_int

_CFG = 40   # stream namespace of this module


def random_signs(seed: int, stream_id: int, shape) -> np.ndarray:
    """int8 tensor of +1 / -1, one fair bit per element."""
    count = int(np.prod(shape))
    words = stream(seed, _CFG, stream_id, (count + 63) // 64)
    bits = np.unpackbits(words.view(np.uint8), bitorder="little")[:count]
    return (bits.astype(np.int8) * 2 - 1).reshape(shape)


def random_bytes(seed: int, stream_id: int, shape) -> np.ndarray:
    """uint8 tensor, uniform (the 8-bit input of a first layer)."""
    count = int(np.prod(shape))
    words = stream(seed, _CFG, stream_id, (count + 7) // 8)
    return words.view(np.uint8)[:count].reshape(shape).copy()


def thresholds(seed: int, stream_id: int, K: int, length: int):
    """(xi, gamma) float32 [K]: thresholds spread over the bulk of the dot product's range
    (standard deviation sqrt(length)), half of them integers of the dot product's parity so
    that the equality case x1 = xi occurs; gamma of both signs, never 0."""
    w = stream(seed, _CFG, stream_id, 3 * K)
    spread = max(1.0, 2.0 * np.sqrt(length))
    xi = (uniform_double(w[:K]) * 2.0 - 1.0) * spread
    exact = uniform_int(w[K:2 * K], 0, 1) == 1
    snapped = np.round(xi / 2.0) * 2.0 + (length % 2)
    xi = np.where(exact, snapped, xi).astype(np.float32)
    mag = 0.25 + uniform_double(w[2 * K:])
    gamma = np.where(uniform_int(w[2 * K:] >> np.uint64(40), 0, 1) == 1, mag, -mag).astype(np.float32)
    return xi, gamma


def batchnorm_parameters(seed: int, stream_id: int, K: int, length: int):
    """(b, mu, sigma, gamma, beta) float64 [K] of an unfused convolution bias + batch norm."""
    w = stream(seed, _CFG, stream_id, 6 * K)
    u = [uniform_double(w[i * K:(i + 1) * K]) for i in range(6)]
    spread = max(1.0, np.sqrt(length))
    b = (u[0] - 0.5) * 4.0
    mu = (u[1] - 0.5) * 2.0 * spread
    sigma = 0.5 + u[2] * spread
    gamma = np.where(u[3] < 0.5, -1.0, 1.0) * (0.1 + u[4])
    beta = (u[5] - 0.5) * 3.0
    return b, mu, sigma, gamma, beta


# Layer shapes in the style of a small single-shot detector's binary trunk at 416 x 416 input
# (each 3x3, stride 1, padding 1, preceded by 2x2 pooling that halves the map; channels double):
# (H = W, C, K).  Seven layers of equal cost up to the 13 x 13 maps, then two wide ones.
DETECTOR_LAYERS = [
    ("conv2", 208, 16, 32), ("conv3", 104, 32, 64), ("conv4", 52, 64, 128), ("conv5", 26, 128, 256),
    ("conv6", 13, 256, 512), ("conv7", 13, 512, 1024), ("conv8", 13, 1024, 1024),
]
# 32 x 32 classifier trunk (3x3, padding 1): (name, H = W, C, K)
CLASSIFIER_LAYERS = [
    ("c1_2", 32, 64, 64), ("c2_1", 16, 64, 128), ("c2_2", 16, 128, 128), ("c3_1", 8, 128, 256), ("c3_2", 8, 256, 256),
    ("c4_1", 4, 256, 512), ("c4_2", 4, 512, 512), ("c5_1", 2, 512, 512),
]


def layer_inputs(seed: int, layer_id: int, N: int, H: int, W: int, C: int, K: int, R: int = 3, S: int = 3):
    """Random activations [N][H][W][C], filters [K][R][S][C] (+1 / -1) and (xi, gamma) of one layer."""
    x = random_signs(seed, 10 * layer_id + 1, (N, H, W, C))
    w = random_signs(seed, 10 * layer_id + 2, (K, R, S, C))
    xi, gamma = thresholds(seed, 10 * layer_id + 3, K, R * S * C)
    return x, w, xi, gamma
