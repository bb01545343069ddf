"""The fused QKV projection of a scorer layer and what follows it on a pass's rows (test oracle).

Alg. 1's scorer call ("else -> prefill") runs, per attention layer, the projection of the
chunk's hidden rows to queries, keys and values, the rotary embedding of queries and keys,
and the append of keys and values to the cache; the paper describes none of it, so this is
the plain definition for the decoder-only model families it trains (Sec. 4.1):

    y[m, n] = sum_k x[m, k] * w[n, k]            (weights stored output-major, as y = x W^T)

with the output columns of a row laid out as [Hq query heads | Hkv key heads | Hkv value
heads], D columns each.  float64 throughout; inputs are bf16 bit patterns widened exactly;
nothing is rounded on the way.
"""
from __future__ import annotations

import numpy as np

from .attention import bf16_bits_to_f64
from .rope import rope_rotate


def qkv_projection(x_bits: np.ndarray, w_bits: np.ndarray, num_q_heads: int, num_kv_heads: int, head_dim: int):
    """x_bits uint16 [rows, hidden], w_bits uint16 [(Hq + 2 Hkv) * D, hidden] ->
    (q [rows, Hq, D], k [rows, Hkv, D], v [rows, Hkv, D]) in float64."""
    x = bf16_bits_to_f64(x_bits)
    w = bf16_bits_to_f64(w_bits)
    rows, hidden = x.shape
    n_out = (num_q_heads + 2 * num_kv_heads) * head_dim
    assert w.shape == (n_out, hidden)
    y = x @ w.T
    q_cols, kv_cols = num_q_heads * head_dim, num_kv_heads * head_dim
    q = y[:, :q_cols].reshape(rows, num_q_heads, head_dim)
    k = y[:, q_cols:q_cols + kv_cols].reshape(rows, num_kv_heads, head_dim)
    v = y[:, q_cols + kv_cols:].reshape(rows, num_kv_heads, head_dim)
    return q, k, v


def qkv_projection_rope(x_bits, w_bits, positions, num_q_heads: int, num_kv_heads: int, head_dim: int,
                        base: float = 10000.0):
    """The projection followed by the rotary embedding of the query and key heads at the rows'
    absolute positions; values pass through.  Returns (q_rot, k_rot, v), float64, unrounded."""
    q, k, v = qkv_projection(x_bits, w_bits, num_q_heads, num_kv_heads, head_dim)
    return rope_rotate(q, positions, base), rope_rotate(k, positions, base), v
