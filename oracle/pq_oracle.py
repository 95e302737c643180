"""CPU oracle for the statically quantized W4A4 linear layer (TEST INFRASTRUCTURE ONLY).

This module is the slow, plain definition of what the HIP library computes.  It is
used by the tests, by the smoke check and by the benchmark's CPU-baseline leg, and by
nothing else: the product path never imports it, and it imports nothing from the
product.  Floating point is fp64 throughout, integer work is int64.

What is defined here, and the passage of the paper each part follows:

  hadamard(h)          Sylvester Hadamard matrix, entries +1/-1 (App. B "Details of
                       Rotation": an orthogonal matrix whose entries are +-1 at one
                       common scale; the common scale is 1/sqrt(h)).
  rotate(x, h)         online rotation of a linear's input, y = x . H_h / sqrt(h) per
                       block of h channels (App. B "Online Rotation", R4-style).
  quantize(y, s)       Eq. 1 in its symmetric form: round to nearest (ties to even),
                       signed 4-bit codes clamped to [-8, 7]; the zero-point of Eq. 1 is
                       the constant 8 and is not stored.  `s` is the static per-tensor
                       step size fixed at calibration (Sec. 3 "Dynamic and Static";
                       Table 1 row O2: activation per-tensor static).
  pack / unpack        two codes per byte, even channel in the low nibble (storage
                       convention of this build; the paper does not fix one).
  gemm_i64(q, wq)      acc[m,n] = sum_k q[m,k] * wq[n,k] in int64 (Sec. 3: low-bit
                       matrix multiplication of quantized weights and activations).
  epilogue(acc,s,sw)   out = fp16(acc * s_x * s_w[n]) (Table 1 row O2: weight
                       per-channel, activation per-tensor; implied by Eq. 1).
  weight_rtn(W)        harness-side preparation: per-output-channel symmetric
                       round-to-nearest 4-bit weights, s_w = rowmax/7 (Table 1:
                       "Weight: per-channel"; stands in for the paper's trained
                       quantizer, which needs data this build does not have).
  calibrate_absmax     harness-side preparation: s_x = max|rotate(x_cal)| / 7 (max-min
                       initialisation of Sec. 3 with gamma = 1, symmetric).
  linear(...)          the whole path in the order above.
  quantize_dynamic     per-token dynamic variant (Table 1 row O1): one step size per
                       row, s[m] = clip * max_k|y[m,k]| / qmax.
  quantize_bits        Eq. 1 symmetric at a general bit-width (8 for the W4A8 setting).
  group_even_odd       storage order of the 8-bit codes (a permutation, no arithmetic): per
                       32 channels the 16 even ones, then the 16 odd ones.
  linear_bits          the whole path with the activation quantizer at `bits` bits.
  quantize_zp, minmax_params, linear_zp
                       Eq. 1 in its general form: X_INT = clamp(round(X/s) + z, 0, 2^N - 1) with
                       s = (gamma max - beta min) / (2^N - 1), z = -round(beta min / s); the stored
                       code is X_INT - 8; the layer adds (8 - z) sum_k w[n,k] to every accumulator.
  silu_mul, rmsnorm    the elementwise producers that static quantization allows to fuse into the
                       quantizer (Sec. 3 "Dynamic and Static"): silu(g) * u and x / rms(x), fp64.
  calibrate_mse        MSE-based grid search for the static per-tensor step (Sec. 3
                       "Initialization of Quantization Parameters"); the paper scores candidates by
                       model block outputs, this build by the tensor's own reconstruction error.
  quantize_groups_dynamic  one step per token and group of consecutive channels (Table 1 row O1, KV cache).
  quantize_heads       per-head static steps (Table 1 row O2, KV cache): the step of channel c is
                       s[c // head_dim]; with rotate() at block = head_dim this is the online R3
                       rotation of the keys followed by their cache quantizer (App. B).

Pins (tests/test_oracle_pins.py): H.H^T = h.I in integers, involution, Parseval,
one-hot and constant rows, block independence, a textbook in-place butterfly written in
the test, on-grid inputs with zero error, exact ties, saturation, pack round trip over
all byte values, brute-force triple loops, the float64 BLAS product of the codes, and
extreme-magnitude accumulators.  No value printed in the paper covers this path (the
paper gives no worked numeric example of rotation, quantizer or product), so parity
with paper-printed numbers is unpinned; the pins are mathematical.
"""

from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_C_SRC = os.path.join(_HERE, "gemm_i64.c")
_C_LIB = os.path.join(_HERE, "libpq_oracle.so")

QMIN, QMAX = -8, 7


# ----------------------------------------------------------------------------- O1
def hadamard(h: int) -> np.ndarray:
    """H_h[i][j] = (-1)^popcount(i & j), 0 <= i, j < h, h a power of two (int8)."""
    if h < 1 or (h & (h - 1)) != 0:
        raise ValueError("h must be a power of two")
    i = np.arange(h, dtype=np.int64)
    both = i[:, None] & i[None, :]
    parity = np.zeros((h, h), dtype=np.int64)
    while np.any(both):
        parity ^= both & 1
        both >>= 1
    return (1 - 2 * parity).astype(np.int8)


# ----------------------------------------------------------------------------- O2
def rotate(x, h: int) -> np.ndarray:
    """y[m, b*h + j] = (sum_i x[m, b*h + i] * H_h[i][j]) / sqrt(h), fp64, dense product."""
    x64 = np.asarray(x, dtype=np.float64)
    M, K = x64.shape
    if h in (0, 1):
        return x64.copy()
    if K % h != 0:
        raise ValueError("h must divide K")
    H = hadamard(h).astype(np.float64)
    blocks = x64.reshape(M, K // h, h)
    y = np.matmul(blocks, H) / np.sqrt(np.float64(h))
    return y.reshape(M, K)


# ----------------------------------------------------------------------------- O3
def quantize(y, s) -> np.ndarray:
    """q = clamp(round_half_even(y / s), -8, 7) as int8; s is a positive scalar."""
    return quantize_bits(y, s, 4)


def quantize_bits(y, s, bits: int) -> np.ndarray:
    """Symmetric Eq. 1 at `bits` bits: codes in [-2^(bits-1), 2^(bits-1) - 1]."""
    t = np.asarray(y, dtype=np.float64) / np.float64(s)
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    return np.clip(np.rint(t), lo, hi).astype(np.int8)


def quantize_heads(y, s_heads, head_dim: int, bits: int = 4) -> np.ndarray:
    """q[t, h*D + j] = clamp(round_half_even(y[t, h*D + j] / s_heads[h]), lo, hi), D = head_dim."""
    y64 = np.asarray(y, dtype=np.float64)
    T, C = y64.shape
    s = np.repeat(np.asarray(s_heads, dtype=np.float64), head_dim)
    assert s.shape == (C,)
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    return np.clip(np.rint(y64 / s[None, :]), lo, hi).astype(np.int8)


def quantize_groups_dynamic(y, group: int, clip: float = 1.0, bits: int = 4):
    """Group-wise dynamic quantization (Table 1 row O1, KV cache): one step per token and group of `group`
    consecutive channels, s[t, g] = fp32(clip * max |y[t, g*group:(g+1)*group]| / qmax), 1 for a group of zeros.
    Returns (codes int8 [T, C], s fp32 [T, C / group])."""
    y64 = np.asarray(y, dtype=np.float64)
    T, C = y64.shape
    qmax = (1 << (bits - 1)) - 1
    yg = y64.reshape(T, C // group, group)
    s = (np.float64(clip) * np.max(np.abs(yg), axis=2) / qmax).astype(np.float32)
    s = np.where(s > 0, s, np.float32(1.0)).astype(np.float32)
    q = np.clip(np.rint(yg / s.astype(np.float64)[:, :, None]), -qmax - 1, qmax).astype(np.int8)
    return q.reshape(T, C), s


def quantize_dynamic(y, clip: float = 1.0, bits: int = 4):
    """Per-token dynamic quantization: s[m] = fp32(clip * max_k |y[m,k]| / qmax).

    Returns (codes int8 [M,K], s fp32 [M]).  A row of zeros gets s = 1 (its codes are
    all zero whatever the step).
    """
    y64 = np.asarray(y, dtype=np.float64)
    qmax = (1 << (bits - 1)) - 1
    amax = np.max(np.abs(y64), axis=1)
    s = (np.float64(clip) * amax / qmax).astype(np.float32)
    s = np.where(s > 0, s, np.float32(1.0)).astype(np.float32)
    t = y64 / s.astype(np.float64)[:, None]
    lo = -(1 << (bits - 1))
    return np.clip(np.rint(t), lo, qmax).astype(np.int8), s


# ----------------------------------------------------------------------------- O4
def pack(q) -> np.ndarray:
    """byte[m, j] = (q[m, 2j] & 0xF) | ((q[m, 2j+1] & 0xF) << 4)."""
    q = np.asarray(q, dtype=np.int8)
    u = q.astype(np.uint8) & 0xF
    return (u[..., 0::2] | (u[..., 1::2] << 4)).astype(np.uint8)


def unpack(b) -> np.ndarray:
    """Inverse of pack: two's-complement nibbles back to int8 in [-8, 7]."""
    b = np.asarray(b, dtype=np.uint8)
    out = np.empty(b.shape[:-1] + (b.shape[-1] * 2,), dtype=np.int8)
    lo = (b & 0xF).astype(np.int16)
    hi = (b >> 4).astype(np.int16)
    out[..., 0::2] = np.where(lo >= 8, lo - 16, lo)
    out[..., 1::2] = np.where(hi >= 8, hi - 16, hi)
    return out


# ----------------------------------------------------------------------------- O5
def group_even_odd(q) -> np.ndarray:
    """out[m, 32g + 16p + j] = q[m, 32g + 2j + p] for p in {0,1}, j in 0..15 (K % 32 == 0)."""
    q = np.asarray(q)
    M, K = q.shape
    assert K % 32 == 0
    return np.ascontiguousarray(q.reshape(M, K // 32, 16, 2).transpose(0, 1, 3, 2).reshape(M, K))


def ungroup_even_odd(b) -> np.ndarray:
    """Inverse of group_even_odd."""
    b = np.asarray(b)
    M, K = b.shape
    assert K % 32 == 0
    return np.ascontiguousarray(b.reshape(M, K // 32, 2, 16).transpose(0, 1, 3, 2).reshape(M, K))


def build_c(force: bool = False) -> str:
    """Compile the C part of the oracle (the int64 product) with gcc; returns the path."""
    stale = (not os.path.exists(_C_LIB)) or os.path.getmtime(_C_LIB) < os.path.getmtime(_C_SRC)
    if force or stale:
        tmp = _C_LIB + ".tmp%d" % os.getpid()
        subprocess.run(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _C_SRC], check=True)
        os.replace(tmp, _C_LIB)
    return _C_LIB


_lib = None


def _c():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_c())
        lib.pqo_gemm_i64.restype = ctypes.c_int
        lib.pqo_gemm_i64.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                     ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p]
        lib.pqo_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the C product uses."""
    return int(_c().pqo_threads())


def gemm_i64(q, wq) -> np.ndarray:
    """acc[m, n] = sum_k (int64) q[m, k] * (int64) wq[n, k]; asserts |acc| < 2^31."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    M, K = q.shape
    N, K2 = wq.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    acc = np.empty((M, N), dtype=np.int64)
    rc = _c().pqo_gemm_i64(q.ctypes.data, wq.ctypes.data, M, N, K, acc.ctypes.data)
    if rc != 0:
        raise OverflowError("accumulator does not fit in int32")
    return acc


# ----------------------------------------------------------------------------- O6
def epilogue(acc, s_x, s_w) -> np.ndarray:
    """out[m, n] = fp16(acc[m, n] * s_x * s_w[n]), product in fp64, one rounding to fp16."""
    a = np.asarray(acc).astype(np.float64)
    sx = np.asarray(s_x, dtype=np.float64)
    if sx.ndim == 1:            # per-token step sizes (dynamic variant)
        sx = sx[:, None]
    sw = np.asarray(s_w, dtype=np.float64)[None, :]
    return (a * sx * sw).astype(np.float16)


# ----------------------------------------------------------------------------- O7
def weight_rtn(W):
    """Per-output-channel symmetric RTN: s_w[n] = fp32(max_k |W[n,k]| / 7), codes int8.

    A row of zeros gets s_w = 1.  Returns (codes [N,K] int8 within [-7,7], s_w fp32 [N]).
    """
    W64 = np.asarray(W, dtype=np.float64)
    s = (np.max(np.abs(W64), axis=1) / 7.0).astype(np.float32)
    s = np.where(s > 0, s, np.float32(1.0)).astype(np.float32)
    codes = np.clip(np.rint(W64 / s.astype(np.float64)[:, None]), QMIN, QMAX).astype(np.int8)
    return codes, s


def calibrate_absmax(x_cal, h: int, bits: int = 4) -> np.float32:
    """s_x = fp32(max |rotate(x_cal, h)| / qmax) over a calibration batch."""
    qmax = (1 << (bits - 1)) - 1
    return np.float32(np.max(np.abs(rotate(x_cal, h))) / qmax)


def quantize_zp(y, s, z: int, bits: int = 4) -> np.ndarray:
    """Eq. 1: X_INT = clamp(round_half_even(y / s) + z, 0, 2^bits - 1); returns X_INT (uint8)."""
    t = np.asarray(y, dtype=np.float64) / np.float64(s)
    return np.clip(np.rint(t) + int(z), 0, (1 << bits) - 1).astype(np.uint8)


def minmax_params(x, gamma: float = 1.0, beta: float = 1.0, bits: int = 4):
    """Eq. 1's parameters from a tensor: s = fp32((gamma max - beta min) / (2^bits - 1)),
    z = -round(beta min / s) clamped to the code range; min is taken as min(x, 0), max as max(x, 0)
    so that zero stays representable."""
    x64 = np.asarray(x, dtype=np.float64)
    hi, lo = max(float(x64.max()), 0.0) * gamma, min(float(x64.min()), 0.0) * beta
    s = np.float32((hi - lo) / ((1 << bits) - 1))
    if not s > 0:
        return np.float32(1.0), 0
    z = int(np.clip(-np.rint(lo / np.float64(s)), 0, (1 << bits) - 1))
    return s, z


def linear_zp(x, wq_packed, s_w, s_x, z: int, h: int):
    """The layer with a zero-point: rotate -> Eq. 1 -> sum_k (X_INT - z) w -> epilogue."""
    y = rotate(x, h)
    u = quantize_zp(y, s_x, z)
    wq = unpack(wq_packed)
    c = u.astype(np.int16) - 8                                   # stored two's-complement codes
    acc = gemm_i64(c.astype(np.int8), wq)
    corr = (8 - int(z)) * wq.astype(np.int64).sum(axis=1)
    return {"y": y, "u": u, "codes": c.astype(np.int8), "acc": acc, "corr": corr,
            "out": epilogue(acc + corr[None, :], np.float32(s_x), s_w)}


def silu_mul(gate, up) -> np.ndarray:
    """silu(gate) * up elementwise, silu(g) = g / (1 + exp(-g)), fp64 (no rounding to fp16)."""
    g = np.asarray(gate, dtype=np.float64)
    return g / (1.0 + np.exp(-g)) * np.asarray(up, dtype=np.float64)


def rmsnorm(x, eps: float) -> np.ndarray:
    """y[m, :] = x[m, :] / sqrt(mean_k x[m, k]^2 + eps), fp64, no learned weight."""
    x64 = np.asarray(x, dtype=np.float64)
    return x64 / np.sqrt(np.mean(x64 * x64, axis=1, keepdims=True) + np.float64(eps))


def calibrate_mse(x_cal, h: int, bits: int = 4, n_grid: int = 50, gamma_min: float = 0.5):
    """Grid search over the clipping factor: gamma_i = 1 - i (1 - gamma_min) / (n_grid - 1),
    s_i = fp32(gamma_i * max|y| / qmax), err_i = sum (y - s_i * Q(y; s_i))^2 with y = rotate(x_cal, h).

    Returns {"best": arg-min index (lowest on a tie), "s": s_best, "s_max": s_0, "gamma": gamma_best,
    "errs": fp64 [n_grid], "steps": fp32 [n_grid]}.  An all-zero tensor gives steps of 1.
    """
    y = rotate(x_cal, h)
    qmax = (1 << (bits - 1)) - 1
    amax = np.max(np.abs(y))
    steps = np.empty(n_grid, dtype=np.float32)
    errs = np.empty(n_grid, dtype=np.float64)
    gammas = np.empty(n_grid, dtype=np.float64)
    for i in range(n_grid):
        gammas[i] = 1.0 - i * (1.0 - np.float64(gamma_min)) / (n_grid - 1)
        s = np.float32(gammas[i] * amax / qmax)
        if not s > 0:
            s = np.float32(1.0)
        steps[i] = s
        q = quantize_bits(y, s, bits).astype(np.float64)
        errs[i] = np.sum((y - np.float64(s) * q) ** 2)
    best = int(np.argmin(errs))
    return {"best": best, "s": steps[best], "s_max": steps[0], "gamma": gammas[best], "errs": errs, "steps": steps}


def calibrate_mse_zp(x_cal, h: int, n_gamma: int = 8, n_beta: int = 8, gamma_min: float = 0.5, beta_min: float = 0.5):
    """Grid search over Eq. 1's parameters: gamma_i on hi = max(y, 0), beta_j on lo = min(y, 0) (linear grids
    from 1 down to the minima; a grid of one point is the factor 1), s = fp32((gamma hi - beta lo) / 15),
    z = clamp(-round(beta lo / s), 0, 15), err = sum (y - s (Q - z))^2; candidate index i * n_beta + j.

    Returns {"best", "s", "z", "errs" fp64 [n], "steps" fp32 [n], "zeros" int [n]}.
    """
    y = rotate(x_cal, h)
    hi, lo = max(float(y.max()), 0.0), min(float(y.min()), 0.0)
    n = n_gamma * n_beta
    steps, zeros, errs = np.empty(n, np.float32), np.empty(n, np.int64), np.empty(n, np.float64)
    for i in range(n_gamma):
        g = 1.0 - i * (1.0 - np.float64(gamma_min)) / (n_gamma - 1) if n_gamma > 1 else 1.0
        for j in range(n_beta):
            b = 1.0 - j * (1.0 - np.float64(beta_min)) / (n_beta - 1) if n_beta > 1 else 1.0
            s = np.float32((g * hi - b * lo) / 15.0)
            if not s > 0:
                s, z = np.float32(1.0), 0
            else:
                z = int(np.clip(-np.rint(b * lo / np.float64(s)), 0, 15))
            c = i * n_beta + j
            steps[c], zeros[c] = s, z
            u = quantize_zp(y, s, z).astype(np.float64)
            errs[c] = np.sum((y - np.float64(s) * (u - z)) ** 2)
    best = int(np.argmin(errs))
    return {"best": best, "s": steps[best], "z": int(zeros[best]), "errs": errs, "steps": steps, "zeros": zeros}


# ----------------------------------------------------------------------------- path
def linear(x, wq_packed, s_w, s_x, h: int, return_all: bool = False):
    """Whole path: rotate -> quantize -> pack -> int64 product -> epilogue."""
    y = rotate(x, h)
    q = quantize(y, s_x)
    xq = pack(q)
    acc = gemm_i64(q, unpack(wq_packed))
    out = epilogue(acc, np.float32(s_x), s_w)
    if return_all:
        return {"y": y, "q": q, "xq": xq, "acc": acc, "out": out}
    return out


def linear_bits(x, wq_packed, s_w, s_x, h: int, bits: int):
    """The path with `bits`-bit static activation codes (8 for the W4A8 setting of Table 3)."""
    y = rotate(x, h)
    q = quantize_bits(y, s_x, bits)
    acc = gemm_i64(q, unpack(wq_packed))
    return {"y": y, "q": q, "acc": acc, "out": epilogue(acc, np.float32(s_x), s_w)}


def linear_dynamic(x, wq_packed, s_w, h: int, clip: float = 1.0, bits: int = 4):
    """Per-token dynamic variant of the path (Table 1 row O1)."""
    y = rotate(x, h)
    q, s = quantize_dynamic(y, clip, bits)
    acc = gemm_i64(q, unpack(wq_packed))
    return {"y": y, "q": q, "s": s, "acc": acc, "out": epilogue(acc, s, s_w)}
