"""Rotary position embedding for one decode step, and the step's append to the key/value cache: the plain definition.

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and nothing in the GPU package); this module imports nothing from
the GPU package either.

arXiv 2401.08294 names the module without a formula: its model-specification table (Section 2, the table of
configurable modules) lists "rope" as the position embedding of the LLaMA-family models.  The published definition
(rotary position embedding) is written out: a head's d components form d/2 pairs; pair i of a vector at position p is
rotated by the angle  p * base^(-2i/d):

    (a, b)  ->  (a cos - b sin,  a sin + b cos)

Two pairings are in use and both are provided: ADJACENT pairs components (2i, 2i+1); HALVES pairs (i, i + d/2).
Keys are stored rotated (each with the angle of its own position), queries are rotated with the current position, and
the values are stored as they are.  Everything in fp64, one rounding to fp16 where a value is stored.
All fp16 inputs and outputs are uint16 bit patterns, like everywhere else in the oracle.
"""
from __future__ import annotations

import numpy as np

ADJACENT, HALVES = 0, 1


def _f(h) -> np.ndarray:
    return np.ascontiguousarray(h, dtype=np.uint16).view(np.float16).astype(np.float64)


def _h(x) -> np.ndarray:
    """fp64 -> fp16 bits, one rounding to nearest-even."""
    return np.asarray(x, dtype=np.float64).astype(np.float16).view(np.uint16)


def angles(position: int, d: int, base: float) -> np.ndarray:
    """The d/2 rotation angles at `position`."""
    i = np.arange(d // 2, dtype=np.float64)
    return float(position) * np.power(float(base), -2.0 * i / d)


def rotate_fp64(x, position: int, base: float, pair_mode: int) -> np.ndarray:
    """x: fp64 [..., d] -> rotated, fp64 (no rounding)."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    ang = angles(position, d, base)
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    if pair_mode == ADJACENT:
        a, b = x[..., 0::2], x[..., 1::2]
        out[..., 0::2] = a * c - b * s
        out[..., 1::2] = a * s + b * c
    elif pair_mode == HALVES:
        a, b = x[..., :d // 2], x[..., d // 2:]
        out[..., :d // 2] = a * c - b * s
        out[..., d // 2:] = a * s + b * c
    else:
        raise ValueError("pair_mode")
    return out


def rope(x16, position: int, base: float, pair_mode: int) -> np.ndarray:
    """fp16 bits in, rotated fp16 bits out (rounded once)."""
    return _h(rotate_fp64(_f(x16), position, base, pair_mode))


def rope_append(q16, k16, v16, position: int, base: float, pair_mode: int, k_cache16, v_cache16):
    """One decode step: returns the rotated queries; writes rotated keys and the values into row `position` of the caches
    ([n_kv_heads][max_seq][d] fp16 bits, modified in place)."""
    k_cache16[:, position, :] = rope(k16, position, base, pair_mode)
    v_cache16[:, position, :] = np.ascontiguousarray(v16, dtype=np.uint16)
    return rope(q16, position, base, pair_mode)
