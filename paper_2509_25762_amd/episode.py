"""Drives one streamed episode through the library (device plumbing only).

The scorer's side of the streaming loop (Alg. 1, generation loop; Sec. 3.1):
the prompt is prefilled once, then every pass appends the chunk's K/V to each
unfinished sequence's cache and lets the chunk attend to prefix + itself.
torch is used for device buffers and row gathers; all arithmetic of the path
runs inside the library.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as ob
from .workload import Episode


def bits_to_device(bits: np.ndarray, device) -> torch.Tensor:
    """uint16 bf16 bit patterns -> int16 device tensor (same bits)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)


class Step:
    """Device inputs of one pass: packed chunk rows of every sequence."""
    __slots__ = ("cu_q", "q_len", "kv_before", "rows", "q", "k", "v", "out")

    def __init__(self, cu_q, q_len, kv_before, rows, q, k, v, out):
        self.cu_q, self.q_len, self.kv_before = cu_q, q_len, kv_before
        self.rows, self.q, self.k, self.v, self.out = rows, q, k, v, out


class StreamedEpisode:
    """All device state of one episode: packed inputs, cache slabs, outputs.

    `chunks[t][i]` is the number of further tokens of sequence i that arrive
    at pass t (pass 0 is normally the prompt).  Sequences keep `slack` spare
    slots after their slab, filled with the 0xFFFF sentinel like every unused
    slot, so that stray writes and out-of-range reads are visible.
    """

    def __init__(self, ep: Episode, chunks: Sequence[Sequence[int]], device="cuda:0", slack: int = 3,
                 use_workspace: bool = True):
        cfg = ep.cfg
        self.ep, self.cfg, self.device = ep, cfg, torch.device(device)
        self.desc = ob.make_desc(cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.softmax_scale)
        B = cfg.batch
        n = ep.prompt_len.astype(np.int64) + ep.resp_len
        self.slot_begin = np.zeros(B + 1, dtype=np.int64)
        np.cumsum(n + slack, out=self.slot_begin[1:])
        self.q_all = bits_to_device(ep.q, self.device)
        self.k_all = bits_to_device(ep.k, self.device)
        self.v_all = bits_to_device(ep.v, self.device)
        total = int(self.slot_begin[-1])
        self.cache_k = torch.full((total, cfg.num_kv_heads, cfg.head_dim), -1, dtype=torch.int16, device=self.device)
        self.cache_v = torch.full_like(self.cache_k, -1)
        self.cache = ob.KVCache(self.cache_k, self.cache_v, self.slot_begin)
        self.out_all = torch.zeros_like(self.q_all)
        self.workspace = None
        if use_workspace:
            nbytes = ob.oppo_workspace_bytes(self.desc, B, int(ep.tok_begin[-1]))
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.steps: List[Step] = []
        done = np.zeros(B, dtype=np.int64)
        for step in chunks:
            q_len = np.asarray(step, dtype=np.int64)
            assert q_len.shape == (B,)
            cu = np.zeros(B + 1, dtype=np.int32)
            np.cumsum(q_len, out=cu[1:])
            rows = np.concatenate([ep.tok_begin[i] + done[i] + np.arange(q_len[i]) for i in range(B)]).astype(np.int64)
            trows = torch.from_numpy(rows).to(self.device)
            self.steps.append(Step(cu, q_len.copy(), done.copy(), trows,
                                   self.q_all[trows].contiguous(), self.k_all[trows].contiguous(),
                                   self.v_all[trows].contiguous(),
                                   torch.zeros((len(rows), cfg.num_q_heads, cfg.head_dim), dtype=torch.int16,
                                               device=self.device)))
            done += q_len
        self.total_done = done

    def reset(self, first_step: int = 0) -> None:
        """Rewinds the host lengths to the state before pass `first_step`."""
        self.cache.kv_len[:] = self.steps[first_step].kv_before if self.steps else 0

    def run_step(self, t: int, stream=None, fused: bool = True) -> None:
        """One pass: the fused call, or append followed by attention (same results)."""
        s = self.steps[t]
        if fused:
            ob.oppo_chunk_step(self.desc, self.cache, s.cu_q, s.q, s.k, s.v, s.out, self.workspace, stream)
        else:
            ob.oppo_kv_append(self.desc, self.cache, s.cu_q, s.k, s.v, stream)
            ob.oppo_chunk_prefill_attn(self.desc, self.cache, s.cu_q, s.q, s.out, self.workspace, stream)

    def run(self, first_step: int = 0, stream=None, fused: bool = True) -> None:
        for t in range(first_step, len(self.steps)):
            self.run_step(t, stream, fused)

    def scatter_outputs(self) -> torch.Tensor:
        """Outputs of all passes at their token rows (int16 bits [T, Hq, D])."""
        for s in self.steps:
            if len(s.rows):
                self.out_all[s.rows] = s.out
        return self.out_all

    def full_prefill(self, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
        """One-shot prefill of every sequence on the device (invariant check)."""
        out = torch.zeros_like(self.q_all)
        cu = self.ep.tok_begin.astype(np.int32)
        ob.oppo_full_prefill_ref(self.desc, cu, self.q_all, self.k_all, self.v_all, out,
                                 self.workspace if workspace is None else workspace)
        return out


def uniform_chunks(prompt_len, resp_len, C: int) -> List[List[int]]:
    """Pass 0 = whole prompts, then the library's schedule for chunk size C."""
    steps = [[int(p) for p in prompt_len]]
    T = int(-(-int(np.max(resp_len)) // C)) if len(resp_len) else 0
    for t in range(T):
        _, q_len, _ = ob.oppo_chunk_schedule(prompt_len, resp_len, C, t)
        steps.append([int(x) for x in q_len])
    return steps
