"""Causal softmax attention, as the definition, in float64 (test oracle).

The streamed scorer of Sec. 3.1 must give exactly what a one-shot prefill
gives (the equivalence argued around Eq. 3), so the oracle is not a model of
any tiling: for a query at absolute position n of a sequence, with q-head h
reading kv-head g = h // (Hq / Hkv),

    S[m]  = s * sum_d Q[n, h, d] * K[m, g, d]        m = 0 .. n
    p[m]  = exp(S[m] - max S) / sum_m exp(S[m] - max S)
    O[n, h, :] = sum_m p[m] * V[m, g, :]

Outputs stay float64 (never rounded to bf16).
"""
from __future__ import annotations

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float64 exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def causal_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray,
                     q_pos: np.ndarray, scale: float,
                     return_weights: bool = False):
    """Attention of a set of query rows of ONE sequence over its keys.

    q      float64 [Tq, Hq, D]   query rows
    k, v   float64 [Tk, Hkv, D]  keys / values of the sequence, row m = token m
    q_pos  int     [Tq]          absolute position n of each query row; the row
                                 sees keys m <= n (needs n < Tk)
    scale  softmax scale s
    Returns O float64 [Tq, Hq, D] (and the weights [Hq, Tq, Tk] if asked).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    q_pos = np.asarray(q_pos, dtype=np.int64)
    Tq, Hq, D = q.shape
    Tk, Hkv, Dk = k.shape
    assert Dk == D and v.shape == k.shape and q_pos.shape == (Tq,)
    assert Hq % Hkv == 0
    if Tq:
        assert q_pos.min() >= 0 and q_pos.max() < Tk, "query position outside the keys"
    G = Hq // Hkv
    s = np.float64(scale)
    visible = np.arange(Tk, dtype=np.int64)[None, :] <= q_pos[:, None]  # [Tq, Tk]
    out = np.empty((Tq, Hq, D), dtype=np.float64)
    weights = np.empty((Hq, Tq, Tk), dtype=np.float64) if return_weights else None
    for h in range(Hq):
        g = h // G
        S = s * (q[:, h, :] @ k[:, g, :].T)           # [Tq, Tk]
        S = np.where(visible, S, -np.inf)
        e = np.exp(S - S.max(axis=1, keepdims=True))
        p = e / e.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ v[:, g, :]
        if return_weights:
            weights[h] = p
    return (out, weights) if return_weights else out


def full_prefill(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float) -> np.ndarray:
    """One-shot causal prefill of a whole sequence: row n sees keys 0..n."""
    return causal_attention(q, k, v, np.arange(q.shape[0]), scale)


def attention_row(q_row: np.ndarray, k: np.ndarray, v: np.ndarray, n: int,
                  h: int, num_q_heads: int, scale: float) -> np.ndarray:
    """Output O[n, h, :] for a single (position, q-head): cost O(n * D).

    q_row float64 [D]; k, v float64 [Tk, Hkv, D].  Used to check sampled rows
    of workloads too large for a full float64 pass.
    """
    Hkv = k.shape[1]
    g = h // (num_q_heads // Hkv)
    S = np.float64(scale) * (k[: n + 1, g, :] @ np.asarray(q_row, dtype=np.float64))
    e = np.exp(S - S.max())
    p = e / e.sum()
    return p @ v[: n + 1, g, :]
