"""CPU oracle for the dense neighbours of the MoE layer -- TEST INFRASTRUCTURE ONLY.

The paper's GPU tasks around the MoE FFN (its section 4.1): the post-attention task (the O
projection, then the MoE FFN) and the pre-attention task (layer norm, then the QKV
projection).  The paper does not write their arithmetic down; the forms below are those of
the models it evaluates (a bias-free linear map, RMS normalisation with a learned scale, a
residual stream), written out in float64 with numpy:

    linear       y = x W^T                         x: dt[T][K], W: dt[N][K]
    add_rmsnorm  s = hidden + delta                (the residual stream, not rounded)
                 x = round_dt( s / sqrt(mean(s^2) + eps) * gamma )

bfloat16 arrays are numpy.uint16 bit patterns, as in the rest of the oracle.
"""
from __future__ import annotations

import numpy as np

from . import round_bf16


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits(v: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 (ties to even) of every double, as bit patterns; one rounding, done by the
    C oracle's scalar routine."""
    r = np.frompyfunc(round_bf16, 1, 1)(np.asarray(v, dtype=np.float64)).astype(np.float64)
    return (r.astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)   # r is exactly representable


def linear(x_bits: np.ndarray, W_bits: np.ndarray) -> np.ndarray:
    """y[t][n] = sum_k x[t][k] * W[n][k], float64."""
    return bf16_bits_to_f64(x_bits) @ bf16_bits_to_f64(W_bits).T


def add_rmsnorm(hidden, delta: np.ndarray, gamma: np.ndarray, eps: float):
    """-> (s float64 [T][H], x bf16 bits [T][H]).  hidden may be None (s = delta)."""
    s = np.asarray(delta, dtype=np.float64) if hidden is None else np.asarray(hidden, np.float64) + np.asarray(delta, np.float64)
    ms = np.mean(s * s, axis=1, keepdims=True)
    x = s / np.sqrt(ms + eps) * np.asarray(gamma, dtype=np.float64)[None, :]
    return s, f64_to_bf16_bits(x)
