"""Seeded synthetic inputs for the five benchmark workloads.

This module only draws numbers.  It holds none of the method's arithmetic and is
the one thing the GPU tests, the benchmark and the CPU oracle checks have in
common: both sides are fed the same arrays.

The paper evaluates on image and language datasets (Sec. 5.2); none of them is
needed for the encode / dot-product path, so tensors with the layer shapes and
value distributions typical of those workloads stand in for them:
activations after a ReLU, He-initialised weights, heavy-tailed small gradients,
log-normal magnitudes, and rows spanning many binades.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 180401526 * 10


def _rng(config: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=BASE_SEED + config, counter=[0, 0, 0, stream]))


def normal(shape, config: int, stream: int = 0, scale: float = 1.0) -> np.ndarray:
    x = _rng(config, stream).standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    return x


def c1_gemm_small(n: int = 256):
    """Config 1: A, B n x n, entries N(0,1)."""
    return normal((n, n), 1, 0), normal((n, n), 1, 1)


def c2_lognormal(n: int = 1 << 26, sigma: float = 3.0) -> np.ndarray:
    """Config 2: n values sign * exp(sigma * Z), Z ~ N(0,1), random signs."""
    g = _rng(2, 0)
    x = g.standard_normal(n, dtype=np.float32)
    x *= np.float32(sigma)
    np.exp(x, out=x)
    s = g.integers(0, 2, size=n, dtype=np.int8)
    x[s == 1] *= np.float32(-1.0)
    return x


def c3_conv_as_gemm(M: int = 100352, K: int = 1152, N: int = 128):
    """Config 3: a 3x3x128 -> 128 convolution on 128 x 28 x 28 outputs, already lowered
    to a matrix product.  X [M,K] = max(0, N(0,1)); W [K,N] ~ N(0, sqrt(2/K));
    dY [M,N] = 1e-3 * Student-t(3)."""
    X = normal((M, K), 3, 0)
    np.maximum(X, 0.0, out=X)
    W = normal((K, N), 3, 1, scale=float(np.sqrt(2.0 / K)))
    g = _rng(3, 2)
    z = g.standard_normal((M, N), dtype=np.float32)
    chi = g.chisquare(3.0, size=(M, N)).astype(np.float32)
    dY = (z / np.sqrt(chi / np.float32(3.0))) * np.float32(1e-3)
    return X, W, dY.astype(np.float32)


def c4_linear(M: int = 4096, K: int = 4096, N: int = 4096):
    """Config 4: dense layer.  X [M,K] ~ N(0,1); W [K,N] ~ N(0, 0.02); dY [M,N] ~ 1e-3 * N(0,1)."""
    return normal((M, K), 4, 0), normal((K, N), 4, 1, scale=0.02), normal((M, N), 4, 2, scale=1e-3)


def c5_wide_range(M: int = 8192, K: int = 8192, N: int = 8192):
    """Config 5: A [M,K], B [K,N]; row i of each is N(0,1) scaled by 2^u_i, u_i uniform in [-20, 20]."""
    out = []
    for stream, (r, c) in enumerate(((M, K), (K, N))):
        x = normal((r, c), 5, stream)
        u = _rng(5, 10 + stream).uniform(-20.0, 20.0, size=(r, 1)).astype(np.float32)
        x *= np.exp2(u)
        out.append(x)
    return out[0], out[1]
