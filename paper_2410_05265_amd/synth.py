"""Seeded synthetic inputs shaped like Llama linears after outlier-token prefixing.

This module only draws random numbers and casts them; it holds none of the method's
arithmetic (no rotation, no quantizer, no product).  Both the CPU oracle's tests and the
GPU harness take their inputs from here so that they see the same bits.

Recipe (all draws from numpy.random.default_rng([seed, stream])):
  stream 0  channel scales  c[K]      = exp(0.5 * g), g ~ N(0,1)   (lognormal(0, 0.5))
  stream 1  activations     X[M,K]    = fp16(randn * c)
  stream 2  calibration     Xcal[T,K] = fp16(randn * c), T = 256 tokens, same c
  stream 3  weights         W[N,K]    = fp16(0.02 * randn)
The activations have per-channel structure but no outlier tokens: removing those is the
post-condition of the paper's prefixing (Sec. 4.2), which is what makes one static
per-tensor step size usable.
"""

from __future__ import annotations

import numpy as np

CAL_TOKENS = 256

# name -> (K, N, hadamard block used when the input is rotated online)
LLAMA2_7B = {"qkv_each": (4096, 4096, 4096), "o": (4096, 4096, 4096),
             "gate": (4096, 11008, 4096), "up": (4096, 11008, 4096),
             "down": (11008, 4096, 128)}
LLAMA3_8B = {"qkv": (4096, 6144, 4096), "o": (4096, 4096, 4096),
             "gate": (4096, 14336, 4096), "up": (4096, 14336, 4096),
             "down": (14336, 4096, 128)}
LLAMA3_70B = {"qkv": (8192, 10240, 8192), "o": (8192, 8192, 8192),
              "gate": (8192, 28672, 8192), "up": (8192, 28672, 8192),
              "down": (28672, 8192, 128)}
TINY = {"tiny": (512, 512, 512)}


def channel_scales(K: int, seed: int = 0) -> np.ndarray:
    g = np.random.default_rng([seed, 0]).standard_normal(K)
    return np.exp(0.5 * g)


def activations(M: int, K: int, seed: int = 0) -> np.ndarray:
    c = channel_scales(K, seed)
    z = np.random.default_rng([seed, 1]).standard_normal((M, K))
    return (z * c).astype(np.float16)


def calibration(K: int, seed: int = 0, tokens: int = CAL_TOKENS) -> np.ndarray:
    c = channel_scales(K, seed)
    z = np.random.default_rng([seed, 2]).standard_normal((tokens, K))
    return (z * c).astype(np.float16)


def weights(N: int, K: int, seed: int = 0) -> np.ndarray:
    z = np.random.default_rng([seed, 3]).standard_normal((N, K), dtype=np.float32)
    return (np.float32(0.02) * z).astype(np.float16)


def random_codes(rows: int, K: int, seed: int = 0, stream: int = 4,
                 lo: int = -8, hi: int = 7) -> np.ndarray:
    """Uniform signed 4-bit codes in [lo, hi], one int8 per element (for product tests)."""
    rng = np.random.default_rng([seed, stream])
    return rng.integers(lo, hi + 1, size=(rows, K), dtype=np.int8)


def random_packed(rows: int, K: int, seed: int = 0, stream: int = 5) -> np.ndarray:
    """Uniform random bytes = uniform pairs of 4-bit codes, [rows, K/2] uint8."""
    rng = np.random.default_rng([seed, stream])
    return rng.integers(0, 256, size=(rows, K // 2), dtype=np.uint8)


def random_scales(N: int, seed: int = 0, stream: int = 6) -> np.ndarray:
    """Positive fp32 per-channel step sizes around 0.02*4/7 (the size RTN gives)."""
    rng = np.random.default_rng([seed, stream])
    return (0.0114 * np.exp(0.1 * rng.standard_normal(N))).astype(np.float32)
