"""Persistent per-sequence KV cache and the streamed episode (test oracle).

Sec. 3.1: the scorer prefills chunk after chunk of a response, each on top of
the chunks it already processed, and the final score rests on the whole
sequence.  The state that carries over is, per sequence, the K/V rows of all
tokens seen so far; with inter-step overlap (Sec. 3.2, Alg. 1 `Buffer.remove`)
an unfinished sequence keeps that state across training iterations.

Layout (the one the library documents): one slab per sequence inside a shared
pool, token-major: slot (slot_begin[i] + m) holds token m of sequence i as
[Hkv, D] bf16 bit patterns.  Append is byte semantics only.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from .attention import bf16_bits_to_f64, causal_attention


class CapacityError(Exception):
    pass


class KVCacheOracle:
    def __init__(self, slot_begin: Sequence[int], num_kv_heads: int, head_dim: int,
                 fill: int = 0xFFFF):
        self.slot_begin = np.asarray(slot_begin, dtype=np.int64)
        assert self.slot_begin.ndim == 1 and self.slot_begin.size >= 1
        assert np.all(np.diff(self.slot_begin) >= 0)
        self.batch = self.slot_begin.size - 1
        total = int(self.slot_begin[-1])
        self.k = np.full((total, num_kv_heads, head_dim), fill, dtype=np.uint16)
        self.v = np.full((total, num_kv_heads, head_dim), fill, dtype=np.uint16)
        self.kv_len = np.zeros(self.batch, dtype=np.int64)

    def capacity(self, i: int) -> int:
        return int(self.slot_begin[i + 1] - self.slot_begin[i])

    def append(self, cu_q: Sequence[int], k_new: np.ndarray, v_new: np.ndarray) -> None:
        """Token j of sequence i's chunk (row cu_q[i]+j of k_new/v_new) goes to
        slot slot_begin[i] + kv_len[i] + j; then kv_len[i] += q_len_i.

        A chunk that does not fit raises CapacityError before anything is
        written or any length changes.
        """
        cu_q = np.asarray(cu_q, dtype=np.int64)
        assert cu_q.shape == (self.batch + 1,) and cu_q[0] == 0
        q_len = np.diff(cu_q)
        assert np.all(q_len >= 0)
        assert k_new.shape[0] == cu_q[-1] and v_new.shape == k_new.shape
        for i in range(self.batch):
            if self.kv_len[i] + q_len[i] > self.capacity(i):
                raise CapacityError(f"sequence {i}: {self.kv_len[i]}+{q_len[i]} > {self.capacity(i)}")
        for i in range(self.batch):
            for j in range(int(q_len[i])):
                slot = int(self.slot_begin[i] + self.kv_len[i] + j)
                self.k[slot] = k_new[cu_q[i] + j]
                self.v[slot] = v_new[cu_q[i] + j]
        self.kv_len += q_len

    def attend(self, cu_q: Sequence[int], q_bits: np.ndarray, scale: float) -> np.ndarray:
        """Attention of each sequence's chunk rows over its cache (which already
        holds the chunk): row j of sequence i is the token at absolute position
        kv_len[i] - q_len_i + j and sees every cached key up to itself.
        Returns float64 [cu_q[B], Hq, D]."""
        cu_q = np.asarray(cu_q, dtype=np.int64)
        q = bf16_bits_to_f64(q_bits)
        out = np.empty(q.shape, dtype=np.float64)
        for i in range(self.batch):
            lo, hi = int(cu_q[i]), int(cu_q[i + 1])
            if hi == lo:
                continue
            n_kv = int(self.kv_len[i])
            assert hi - lo <= n_kv
            b = int(self.slot_begin[i])
            k = bf16_bits_to_f64(self.k[b:b + n_kv])
            v = bf16_bits_to_f64(self.v[b:b + n_kv])
            pos = n_kv - (hi - lo) + np.arange(hi - lo)
            out[lo:hi] = causal_attention(q[lo:hi], k, v, pos, scale)
        return out


def stream_episode(q_bits: List[np.ndarray], k_bits: List[np.ndarray], v_bits: List[np.ndarray],
                   chunks: List[List[int]], scale: float, capacity_slack: int = 0):
    """Stream every sequence through a cache in the given chunks.

    q_bits/k_bits/v_bits: per sequence, all of its tokens [N_i, H, D] (uint16).
    chunks[t][i]: how many further tokens of sequence i arrive at pass t (0 =
    the sequence sits this pass out); over all passes they sum to N_i.
    Returns (outputs per sequence float64 [N_i, Hq, D], the cache).
    """
    B = len(q_bits)
    n = [int(x.shape[0]) for x in q_bits]
    slot_begin = np.zeros(B + 1, dtype=np.int64)
    for i in range(B):
        slot_begin[i + 1] = slot_begin[i] + n[i] + capacity_slack
    Hkv, D = k_bits[0].shape[1], k_bits[0].shape[2]
    cache = KVCacheOracle(slot_begin, Hkv, D)
    outs = [np.empty(q_bits[i].shape, dtype=np.float64) for i in range(B)]
    done = [0] * B
    for step in chunks:
        assert len(step) == B
        cu_q = np.zeros(B + 1, dtype=np.int64)
        for i in range(B):
            cu_q[i + 1] = cu_q[i] + step[i]
        def gather(src):
            parts = [src[i][done[i]:done[i] + step[i]] for i in range(B)]
            return np.concatenate(parts, axis=0)
        cache.append(cu_q, gather(k_bits), gather(v_bits))
        o = cache.attend(cu_q, gather(q_bits), scale)
        for i in range(B):
            outs[i][done[i]:done[i] + step[i]] = o[cu_q[i]:cu_q[i + 1]]
            done[i] += step[i]
    assert done == n, "chunks do not cover every token"
    return outs, cache
