"""Rotary position embedding of a pass's query and key rows (test oracle).

The scorer is a decoder-only transformer of the Llama / Qwen family (Sec. 4.1),
whose attention layers rotate every query and key row by an angle that grows
with the row's absolute position before the keys enter the cache.  The paper
itself says nothing about it; this is the published definition (Su et al.,
"RoFormer", Sec. 3.2 and 3.4.2) in the pairing those model families use:

  theta_i = base ** (-2 i / D),                  i = 0 .. D/2 - 1
  (x_i, x_{i + D/2})  ->  (x_i cos(p theta_i) - x_{i + D/2} sin(p theta_i),
                           x_{i + D/2} cos(p theta_i) + x_i sin(p theta_i))

for a row at absolute position p.  With streamed chunks p = kv_before + j for
row j of a sequence's chunk, which is what makes the rotated keys of earlier
chunks reusable from the cache (Sec. 3.1).  float64 throughout.
"""
from __future__ import annotations

import numpy as np


def rope_rotate(x: np.ndarray, pos: np.ndarray, base: float = 10000.0) -> np.ndarray:
    """x: float64 [n, H, D]; pos: absolute position of each of the n rows."""
    x = np.asarray(x, dtype=np.float64)
    pos = np.asarray(pos, dtype=np.float64)
    n, H, D = x.shape
    assert D % 2 == 0 and pos.shape == (n,)
    half = D // 2
    theta = np.asarray([base ** (-2.0 * i / D) for i in range(half)], dtype=np.float64)
    out = np.empty_like(x)
    for r in range(n):
        ang = pos[r] * theta
        c, s = np.cos(ang), np.sin(ang)
        for h in range(H):
            a, b = x[r, h, :half], x[r, h, half:]
            out[r, h, :half] = a * c - b * s
            out[r, h, half:] = b * c + a * s
    return out


def pass_positions(kv_before, q_len) -> np.ndarray:
    """Absolute positions of a pass's packed rows: kv_before[i] + j for row j of sequence i."""
    parts = [int(k) + np.arange(int(q)) for k, q in zip(kv_before, q_len)]
    return np.concatenate(parts) if parts else np.zeros(0, dtype=np.int64)
