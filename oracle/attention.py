"""Plain definition of one decode step of grouped-query attention over a key/value cache, for the GPU kernel's parity tests.

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and by nothing in the GPU package); imports nothing from it either.

arXiv 2401.08294, section "Grouped-query attention": with H query heads in G groups, query head i attends with the
keys and values of its group j, head_i = Attention(Q_i, K^j, V^j); H = G is plain multi-head attention.  Attention is
scaled dot-product attention (the paper's citation of Vaswani et al.): softmax(q K^T * scale) V.  A decode step has
one query position, and every cached position is visible to it.  Written out in fp64, on fp16 inputs given as uint16
bit patterns like everywhere else in the oracle:

  q        [n_heads][head_dim]
  k_cache  [n_kv_heads][max_seq][head_dim]      (only positions < seq_len are read)
  v_cache  [n_kv_heads][max_seq][head_dim]
  out      [n_heads][head_dim]   fp64
"""
from __future__ import annotations

import numpy as np


def _f(h) -> np.ndarray:
    return np.ascontiguousarray(h, dtype=np.uint16).view(np.float16).astype(np.float64)


def gqa_decode(q16_bits, k16_bits, v16_bits, seq_len: int, scale: float) -> np.ndarray:
    q, k, v = _f(q16_bits), _f(k16_bits), _f(v16_bits)
    n_heads, d = q.shape
    n_kv = k.shape[0]
    assert n_heads % n_kv == 0 and k.shape == v.shape and k.shape[2] == d and 1 <= seq_len <= k.shape[1]
    per_group = n_heads // n_kv                       # query heads that share one key/value head
    out = np.zeros((n_heads, d), np.float64)
    for i in range(n_heads):
        j = i // per_group
        s = (k[j, :seq_len] @ q[i]) * scale           # one score per cached position
        p = np.exp(s - np.max(s))
        p /= np.sum(p)
        out[i] = p @ v[j, :seq_len]
    return out
