"""Plain definitions of the modules that sit around a linear layer in one decode step, for the fused GEMV's parity tests.

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and nothing in the GPU package); this module imports nothing from
the GPU package either.

arXiv 2401.08294 names these modules without formulas: its model-specification table (Section 2, the table of
configurable modules) lists "rms" as the normalization function and "silu" as the activation function of the
LLaMA-family models its decode step (Section 5, ``Infer()``) runs.  So the textbook definitions are written out:

  rms normalization  y_k = x_k * g_k / sqrt(mean_j x_j^2 + eps)
  silu               silu(a) = a / (1 + exp(-a))
  gated feed-forward input  v_k = silu(a_k) * b_k      (a: "gate" projection, b: "up" projection)
  residual           out_n = (W v)_n + r_n
  gated pair         out_n = silu(scale (W_gate v)_n) * (scale (W_up v)_n)      (the gate applied where its two
                     projections are produced, before either is stored)

The definitions that parity is judged by are the unsplit ones - ``rms_linear``, ``silu_linear``, ``gated_rms`` - evaluated
in fp64 from the fp16 inputs with no rounding anywhere in between: they know nothing of how a kernel orders the work.

A second, narrower set (``gain``, ``rms_scale``, ``silu_mul``, ``fused_gemv``, ``gated_gemv``) states one particular
evaluation order with its fp16 roundings - normalization as fp16(x_k g_k) in front of the matrix and the scalar
1 / sqrt(mean x^2 + eps) behind it (the scalar commutes with the matrix product), the gated input rounded to fp16 before the
product.  Tests use it only as an additional, tighter check of where a kernel's error comes from; it decides nothing.
All fp16 inputs and outputs are uint16 bit patterns, like everywhere else in the oracle.
"""
from __future__ import annotations

import numpy as np


def _f(h) -> np.ndarray:
    return np.ascontiguousarray(h, dtype=np.uint16).view(np.float16).astype(np.float64)


def _h(x) -> np.ndarray:
    """fp64 -> fp16 bits, one rounding to nearest-even."""
    return np.asarray(x, dtype=np.float64).astype(np.float16).view(np.uint16)


# ---- the definitions (no intermediate rounding) ---------------------------------------------------------------------

def rms_norm(x16_bits, g16_bits, eps: float) -> np.ndarray:
    """x_k g_k / sqrt(mean_j x_j^2 + eps) in fp64."""
    x = _f(x16_bits)
    return x * _f(g16_bits) / np.sqrt(np.mean(x * x) + eps)


def rms_linear(w16_bits, x16_bits, g16_bits, eps: float, residual16_bits=None) -> np.ndarray:
    """W' rms_norm(x; g, eps) (+ residual) in fp64: a linear layer behind an rms normalization."""
    y = _f(w16_bits) @ rms_norm(x16_bits, g16_bits, eps)
    if residual16_bits is not None:
        y = y + _f(residual16_bits)
    return y


def silu_linear(w16_bits, a16_bits, b16_bits, residual16_bits=None) -> np.ndarray:
    """W' (silu(a) * b) (+ residual) in fp64: the last projection of a gated feed-forward from its two hidden vectors."""
    y = _f(w16_bits) @ (silu(_f(a16_bits)) * _f(b16_bits))
    if residual16_bits is not None:
        y = y + _f(residual16_bits)
    return y


def gated_rms(w_gate16_bits, w_up16_bits, x16_bits, g16_bits=None, eps: float = 0.0) -> np.ndarray:
    """silu(W_gate' n) * (W_up' n) in fp64, n = rms_norm(x; g, eps), or n = x when g16_bits is None."""
    n = _f(x16_bits) if g16_bits is None else rms_norm(x16_bits, g16_bits, eps)
    return silu(_f(w_gate16_bits) @ n) * (_f(w_up16_bits) @ n)


# ---- one evaluation order with its fp16 roundings (secondary checks only) -------------------------------------------

def rms_scale(x16_bits, eps: float) -> float:
    """1 / sqrt(mean_k x_k^2 + eps), fp64."""
    x = _f(x16_bits)
    return float(1.0 / np.sqrt(np.mean(x * x) + eps))


def gain(x16_bits, g16_bits) -> np.ndarray:
    """fp16(x_k * g_k): the product of two fp16 numbers is exact in fp64, so this is a single rounding."""
    return _h(_f(x16_bits) * _f(g16_bits))


def silu(a) -> np.ndarray:
    a = np.asarray(a, dtype=np.float64)
    return a / (1.0 + np.exp(-a))


def silu_mul(a16_bits, b16_bits) -> np.ndarray:
    """fp16(silu(a_k) * b_k)."""
    return _h(silu(_f(a16_bits)) * _f(b16_bits))


def fused_gemv(w16_bits, v16_bits, scale: float = 1.0, residual16_bits=None) -> np.ndarray:
    """scale * (W' v) + residual in fp64 (W' fp16 [rows][cols], v fp16 [cols], residual fp16 [rows] or None)."""
    w = _f(w16_bits)
    y = scale * (w @ _f(v16_bits))
    if residual16_bits is not None:
        y = y + _f(residual16_bits)
    return y


def gated_gemv(w_gate16_bits, w_up16_bits, v16_bits, scale: float = 1.0) -> np.ndarray:
    """silu(scale * (W_gate' v)) * (scale * (W_up' v)) in fp64: the gated feed-forward's hidden vector from its two
    projections, with no rounding in between."""
    v = _f(v16_bits)
    return silu(scale * (_f(w_gate16_bits) @ v)) * (scale * (_f(w_up16_bits) @ v))
