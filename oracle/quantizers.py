"""CPU oracle for the quantisers (Preliminaries, Eq. 1a-1c) and the aggregated quantisation
functions of the bitwidth search (Sec. 4.1: Eq. 6 for weights, Eq. 7 for activations, Eq. 8 for
the stochastic coefficients).  TEST INFRASTRUCTURE ONLY, like the rest of this package.

Plain numpy in float64, each function the formula as written.  The one exception is the
activation level, where a rounding decides an integer: that decision is taken in single
precision in a fixed order (bd_oracle.c, oracle_activation_levels), the same on both sides;
``quantize_activations_f64`` is the float64 definition it is pinned against.

Readings of the paper (it is silent or garbled on these):
* round() is round half up: floor(v + 0.5) (stated below Eq. 1c).
* all-zero weights: max|tanh W| = 0 makes Eq. 1a 0/0; the normalised value is taken as 0, i.e.
  every weight sits at 1/2 before rounding.
* Eq. 8 as printed has the division by tau outside exp(); the Gumbel-softmax it cites divides
  the logits: coefficient_i = exp((log p_i + g_i)/tau) / sum_j exp((log p_j + g_j)/tau).
"""
from __future__ import annotations

import ctypes

import numpy as np


def quantize_b(x, b: int):
    """Eq. 1c: quantize_b(x) = round((2^b - 1) x) / (2^b - 1), round half up."""
    n = (1 << b) - 1
    return np.floor(n * np.asarray(x, dtype=np.float64) + 0.5) / n


def _normalised_weights(W):
    t = np.tanh(np.asarray(W, dtype=np.float64))
    m = np.max(np.abs(t)) if t.size else 0.0
    if m == 0.0:
        return np.full(t.shape, 0.5)
    return t / (2.0 * m) + 0.5                      # in [0, 1]


def weight_levels(W, b: int):
    """Integer level q in [0, 2^b - 1] inside Eq. 1a: round((2^b - 1) (tanh W / (2 max|tanh W|) + 1/2))."""
    n = (1 << b) - 1
    return np.floor(n * _normalised_weights(W) + 0.5).astype(np.uint8)


def quantize_weights(W, b: int):
    """Eq. 1a: W_hat = 2 quantize_b(tanh W / (2 max|tanh W|) + 1/2) - 1, in [-1, 1]."""
    return 2.0 * quantize_b(_normalised_weights(W), b) - 1.0


def quantize_activations_f64(X, alpha: float, b: int):
    """Eq. 1b in float64: X_hat = alpha quantize_b(clip(X, 0, alpha) / alpha)."""
    X = np.asarray(X, dtype=np.float64)
    return alpha * quantize_b(np.clip(X, 0.0, alpha) / alpha, b)


def activation_levels(X, alpha: float, b: int):
    """Integer level of Eq. 1b-1c, decided in single precision (see the module header)."""
    from . import _load
    x = np.ascontiguousarray(X, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint8)
    _load().oracle_activation_levels(x.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), x.size,
                                     ctypes.c_float(alpha), b, out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)))
    return out


def quantize_activations(X, alpha: float, b: int):
    """Eq. 1b with the level decided as in activation_levels: alpha * level / (2^b - 1) (float64)."""
    return float(np.float32(alpha)) * activation_levels(X, alpha, b).astype(np.float64) / ((1 << b) - 1)


def softmax(r):
    """exp(r_i) / sum_j exp(r_j) (the coefficients of Eq. 5-7)."""
    r = np.asarray(r, dtype=np.float64)
    e = np.exp(r - np.max(r))
    return e / e.sum()


def gumbel_softmax(r, g, tau: float):
    """Eq. 8: p = softmax(r); coefficient_i = exp((log p_i + g_i)/tau) / sum_j exp((log p_j + g_j)/tau),
    g the Gumbel(0,1) samples (an input: the caller draws them)."""
    p = softmax(r)
    y = (np.log(p) + np.asarray(g, dtype=np.float64)) / tau
    e = np.exp(y - np.max(y))
    return e / e.sum()


def _coefficients(strengths, gumbel, tau):
    return softmax(strengths) if gumbel is None else gumbel_softmax(strengths, gumbel, tau)


def aggregate_weights(W, bits, strengths, gumbel=None, tau: float = 1.0):
    """Eq. 6 (Eq. 8 with gumbel): sum_i coefficient_i * W_hat^{b_i}, one meta weight tensor."""
    c = _coefficients(strengths, gumbel, tau)
    out = np.zeros(np.shape(W), dtype=np.float64)
    for ci, b in zip(c, bits):
        out += ci * quantize_weights(W, b)
    return out


def aggregate_activations(X, alpha: float, bits, strengths, gumbel=None, tau: float = 1.0):
    """Eq. 7, activation factor: sum_i coefficient_i * X_hat^{b_i}."""
    c = _coefficients(strengths, gumbel, tau)
    out = np.zeros(np.shape(X), dtype=np.float64)
    for ci, b in zip(c, bits):
        out += ci * quantize_activations(X, alpha, b)
    return out
