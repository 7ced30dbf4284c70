"""Seeded synthetic inputs shaped like the workloads of the quantized decode step.

This module holds no quantization or matmul arithmetic: it only draws numbers.  It is the one
module that both the CPU oracle's tests and the GPU path's tests/benchmark may share, so that both
sides see bit-identical inputs.  Everything is generated on the host with numpy's PCG64
(`default_rng(seed)`), in float32, and activations are then rounded to fp16.

Stand-ins: the paper evaluates on trained LLaMA-2 / Bloom / Falcon weights; here weights are
zero-mean Gaussians with the usual initialisation spread (standard deviation 0.02, or 0.015 for the
70B shapes), optionally with a small fraction of entries multiplied by 10 to stretch block ranges.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 2401082940

# (rows N, cols K) of the linears of one Llama-2 decoder layer: Y = X W^T, W is [N][K]
LLAMA2_7B_LAYER = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                   ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
LLAMA2_70B_SHAPES = [("attn", 8192, 8192), ("gate_up", 28672, 8192), ("down", 8192, 28672)]


def weights(rows: int, cols: int, sigma: float = 0.02, seed: int = BASE_SEED,
            outlier_prob: float = 0.0, outlier_scale: float = 10.0) -> np.ndarray:
    """fp32 [rows][cols] ~ N(0, sigma^2); each entry independently scaled by `outlier_scale` with prob. `outlier_prob`."""
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(sigma)
    if outlier_prob > 0.0:
        mask = rng.random((rows, cols), dtype=np.float32) < np.float32(outlier_prob)
        w = np.where(mask, w * np.float32(outlier_scale), w).astype(np.float32)
    return np.ascontiguousarray(w)


def activations(batch: int, cols: int, seed: int = BASE_SEED + 1) -> np.ndarray:
    """fp16 [batch][cols] ~ N(0, 1), returned as a float16 array."""
    rng = np.random.default_rng(seed)
    return np.ascontiguousarray(rng.standard_normal((batch, cols), dtype=np.float32).astype(np.float16))


def sample_rows(rows: int, count: int, seed: int = BASE_SEED + 2) -> np.ndarray:
    """`count` distinct sorted row indices, always including the first and last row."""
    rng = np.random.default_rng(seed)
    count = min(count, rows)
    idx = set([0, rows - 1]) if rows > 1 else {0}
    while len(idx) < count:
        idx.add(int(rng.integers(0, rows)))
    return np.array(sorted(idx), dtype=np.int64)
