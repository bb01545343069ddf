"""Seeded synthetic workloads for the chunked-prefill attention path.

This module only draws inputs (lengths and bf16 Q/K/V tensors) and counts the
algorithmic work of a workload.  It contains none of the attention arithmetic
and imports neither the CPU oracle nor the HIP binding, so both sides of a
parity test can be fed from it.

The lengths stand in for the rollouts of the paper's PPO runs (Sec. 4.1): most
responses are short and a few are much longer (Sec. 2.2, long-tailed response
lengths), which is modelled with a clipped log-normal.  Chunk sizes bracket the
ones the paper discusses (Sec. 3.1: 128/256/512 candidates; Sec. 4.3 sweep).

Recipe (fixed so that every run sees the same numbers):
  rng = numpy.random.default_rng(seed)                       (PCG64)
  draw order: prompt lengths, response normals, straggler indices
  tensors of sequence i: default_rng([seed, i, tensor_id]) with tensor_id
  0/1/2 = Q/K/V, standard_normal(float32), rounded to nearest-even bf16.
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Tuple

import numpy as np


@dataclasses.dataclass(frozen=True)
class Config:
    index: int
    name: str
    seed: int
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    chunk: int
    prompt: Tuple  # ("uniform", lo, hi) inclusive | ("fixed", n)
    response: Tuple  # ("fixed", n) | ("lognormal", median, sigma, lo, hi)
    straggler_frac: float = 0.0
    straggler_len: int = 0

    @property
    def softmax_scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads


CONFIGS: Dict[int, Config] = {
    1: Config(1, "tiny", 20250926, 4, 4, 4, 64, 32, ("uniform", 32, 64), ("fixed", 128)),
    2: Config(2, "llama3-8b-shape", 20250927, 64, 32, 8, 128, 256,
              ("uniform", 256, 1024), ("lognormal", 512, 0.8, 16, 4096)),
    3: Config(3, "small-chunk", 20250928, 256, 32, 8, 128, 64,
              ("uniform", 512, 2048), ("lognormal", 256, 1.0, 8, 2048)),
    4: Config(4, "long-tail", 20250929, 32, 32, 8, 128, 512,
              ("fixed", 2048), ("lognormal", 1024, 1.0, 64, 8192), 0.05, 8192),
    5: Config(5, "70b-shape", 20250930, 16, 64, 8, 128, 1024,
              ("uniform", 1024, 4096), ("lognormal", 2048, 0.9, 128, 12288)),
}


def draw_lengths(cfg: Config) -> Tuple[np.ndarray, np.ndarray]:
    """Prompt lengths P[B] and final response lengths R[B] (int32)."""
    rng = np.random.default_rng(cfg.seed)
    B = cfg.batch
    if cfg.prompt[0] == "uniform":
        P = rng.integers(cfg.prompt[1], cfg.prompt[2], size=B, endpoint=True)
    else:
        P = np.full(B, cfg.prompt[1])
    if cfg.response[0] == "fixed":
        R = np.full(B, cfg.response[1])
    else:
        _, median, sigma, lo, hi = cfg.response
        z = rng.standard_normal(B)
        R = np.clip(np.rint(np.exp(math.log(median) + sigma * z)), lo, hi)
    R = R.astype(np.int64)
    if cfg.straggler_frac > 0.0:
        n = int(math.ceil(cfg.straggler_frac * B))
        idx = rng.choice(B, size=n, replace=False)
        R[idx] = cfg.straggler_len
    return P.astype(np.int32), R.astype(np.int32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the 16 bits.

    Inputs here are finite normals, so no NaN handling is needed.
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def draw_tensor_bits(seed: int, seq: int, tensor_id: int, shape) -> np.ndarray:
    """bf16 bits (uint16) of an N(0,1) tensor of sequence `seq`."""
    rng = np.random.default_rng([seed, seq, tensor_id])
    return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))


def draw_sequence(cfg: Config, seq: int, n_tokens: int):
    """(q_bits [N,Hq,D], k_bits [N,Hkv,D], v_bits [N,Hkv,D]) of one sequence."""
    q = draw_tensor_bits(cfg.seed, seq, 0, (n_tokens, cfg.num_q_heads, cfg.head_dim))
    k = draw_tensor_bits(cfg.seed, seq, 1, (n_tokens, cfg.num_kv_heads, cfg.head_dim))
    v = draw_tensor_bits(cfg.seed, seq, 2, (n_tokens, cfg.num_kv_heads, cfg.head_dim))
    return q, k, v


@dataclasses.dataclass
class Episode:
    """All inputs of one streamed episode, packed sequence after sequence.

    q/k/v hold every token of every sequence (prompt then response) at rows
    [tok_begin[i], tok_begin[i+1]).
    """
    cfg: Config
    prompt_len: np.ndarray  # int32 [B]
    resp_len: np.ndarray  # int32 [B]
    tok_begin: np.ndarray  # int64 [B+1]
    q: np.ndarray  # uint16 [T, Hq, D]
    k: np.ndarray  # uint16 [T, Hkv, D]
    v: np.ndarray  # uint16 [T, Hkv, D]

    @property
    def num_steps(self) -> int:
        return int(-(-int(self.resp_len.max()) // self.cfg.chunk))


def build_episode(cfg: Config, threads: int = 8,
                  lengths: Optional[Tuple[np.ndarray, np.ndarray]] = None) -> Episode:
    P, R = lengths if lengths is not None else draw_lengths(cfg)
    n = P.astype(np.int64) + R.astype(np.int64)
    tok_begin = np.zeros(cfg.batch + 1, dtype=np.int64)
    np.cumsum(n, out=tok_begin[1:])
    T = int(tok_begin[-1])
    q = np.empty((T, cfg.num_q_heads, cfg.head_dim), dtype=np.uint16)
    k = np.empty((T, cfg.num_kv_heads, cfg.head_dim), dtype=np.uint16)
    v = np.empty((T, cfg.num_kv_heads, cfg.head_dim), dtype=np.uint16)

    def fill(job):
        i, tid = job
        dst = (q, k, v)[tid]
        lo, hi = int(tok_begin[i]), int(tok_begin[i + 1])
        dst[lo:hi] = draw_tensor_bits(cfg.seed, i, tid, (hi - lo,) + dst.shape[1:])

    jobs = [(i, tid) for i in range(cfg.batch) for tid in range(3)]
    if threads > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, jobs))
    else:
        for j in jobs:
            fill(j)
    return Episode(cfg, P, R, tok_begin, q, k, v)


# ---------------------------------------------------------------------------
# Work accounting (counts only; no attention arithmetic).
# ---------------------------------------------------------------------------

def step_work(cfg: Config, kv_before: np.ndarray, q_len: np.ndarray) -> Dict[str, float]:
    """Algorithmic FLOPs and bytes of one chunk step.

    FLOPs: QK^T and PV, 2 per multiply-add, causally visible pairs only.
    KV-read bytes: each active (sequence, kv-head) reads its K and V once.
    """
    kvb = kv_before.astype(np.float64)
    ql = q_len.astype(np.float64)
    D, Hq, Hkv = cfg.head_dim, cfg.num_q_heads, cfg.num_kv_heads
    pairs = float(np.sum(ql * kvb + ql * (ql + 1.0) / 2.0))
    active = q_len > 0
    kv_after = (kv_before + q_len)[active].astype(np.float64)
    rows = float(ql.sum())
    return {
        "flops": 4.0 * D * Hq * pairs,
        "kv_read_bytes": float(kv_after.sum()) * Hkv * D * 2 * 2,
        "qo_bytes": 2.0 * rows * Hq * D * 2,
        "append_bytes": 2.0 * rows * Hkv * D * 2 * 2,
        "rows": rows,
        "active": float(active.sum()),
    }


def episode_work(cfg: Config, steps) -> List[Dict[str, float]]:
    """Per-step work of an episode; `steps` yields (kv_before[B], q_len[B])
    as produced by the chunk scheduler of whichever side is being measured."""
    return [step_work(cfg, np.asarray(kvb), np.asarray(ql)) for kvb, ql in steps]
