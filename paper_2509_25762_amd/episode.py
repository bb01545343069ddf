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
        align = self.slot_align
        np.cumsum((n + slack + align - 1) // align * align, out=self.slot_begin[1:])
        self.q_all = bits_to_device(ep.q, self.device)
        self.k_all = bits_to_device(ep.k, self.device)
        self.v_all = bits_to_device(ep.v, self.device)
        self._make_cache(int(self.slot_begin[-1]))
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

    slot_align = 1   # slabs start on multiples of this many slots

    def _make_cache(self, total: int) -> None:
        cfg = self.cfg
        self.cache_k = torch.full((total, cfg.num_kv_heads, cfg.head_dim), -1, dtype=torch.int16, device=self.device)
        self.cache_v = torch.full_like(self.cache_k, -1)
        self.cache = ob.KVCache(self.cache_k, self.cache_v, self.slot_begin)

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


class StreamedEpisodeFp8(StreamedEpisode):
    """The same episode through the cache of 8-bit codes (append + attention calls; every unused
    byte starts as 0xFF).  full_prefill is not available: the one-shot reference has no cache."""
    slot_align = 64

    def __init__(self, ep: Episode, chunks: Sequence[Sequence[int]], k_scale: float, v_scale: float, **kw):
        self.k_scale, self.v_scale = float(k_scale), float(v_scale)
        super().__init__(ep, chunks, **kw)

    def _make_cache(self, total: int) -> None:
        cfg = self.cfg
        self.cache_k = torch.full((total, cfg.num_kv_heads, cfg.head_dim), 0xFF, dtype=torch.uint8, device=self.device)
        self.cache_v = torch.full((total // 64, cfg.num_kv_heads, cfg.head_dim, 64), 0xFF, dtype=torch.uint8,
                                  device=self.device)
        self.cache = ob.KVCacheFp8(self.cache_k, self.cache_v, self.slot_begin, self.k_scale, self.v_scale)

    def run_step(self, t: int, stream=None, fused: bool = False) -> None:
        if fused:
            raise ValueError("the 8-bit cache has no fused call: append, then attend")
        s = self.steps[t]
        ob.oppo_kv_append_fp8(self.desc, self.cache, s.cu_q, s.k, s.v, stream)
        ob.oppo_chunk_prefill_attn_fp8(self.desc, self.cache, s.cu_q, s.q, s.out, self.workspace, stream)

    def run(self, first_step: int = 0, stream=None, fused: bool = False) -> None:
        super().run(first_step, stream, fused)

    def full_prefill(self, workspace=None):
        raise NotImplementedError("no 8-bit one-shot reference")


def uniform_chunks(prompt_len, resp_len, C: int) -> List[List[int]]:
    """Pass 0 = whole prompts, then the library's schedule for chunk size C."""
    steps = [[int(p) for p in prompt_len]]
    T = int(-(-int(np.max(resp_len)) // C)) if len(resp_len) else 0
    for t in range(T):
        _, q_len, _ = ob.oppo_chunk_schedule(prompt_len, resp_len, C, t)
        steps.append([int(x) for x in q_len])
    return steps


class BufferedPass:
    """Device inputs of one scorer pass of a BufferedRun (rows packed in slot order)."""
    __slots__ = ("iteration", "kind", "ids", "kv_before", "q_len", "cu_q", "rows", "q", "k", "v", "out")

    def __init__(self, **kw):
        for name, value in kw.items():
            setattr(self, name, value)


class BufferedRun:
    """Alg. 1 with inter-step overlap over a synthetic dataset (device plumbing only).

    The library's buffer state machine (oppo_sched_*) decides who is served when,
    its slot pool (oppo_pool_*) gives each sequence in the buffer one of B + delta
    cache slabs, and every pass is one oppo_chunk_step over all slots (sequences
    that sit the pass out have no rows).  The "actor" is simulated: the final
    response lengths of the dataset are known, a sequence produces min(C, what is
    left) tokens per pass.  Sec. 3.2, Alg. 1.

    The host logic runs once, in __init__, against a scheduler and a pool of its
    own (lengths advanced by hand), to gather every pass's input rows in advance;
    run() then replays acquisitions, passes and releases against a fresh pool, so
    that a timed run contains library calls only.
    """

    def __init__(self, ep: Episode, B: int, delta: int, C: int, device="cuda:0", slack: int = 3,
                 use_workspace: bool = True, max_iterations: Optional[int] = None):
        cfg = ep.cfg
        self.ep, self.cfg, self.device = ep, cfg, torch.device(device)
        self.B, self.delta, self.C = B, delta, C
        self.desc = ob.make_desc(cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.softmax_scale)
        n = ep.prompt_len.astype(np.int64) + ep.resp_len
        self.n_slots = B + delta
        self.capacity = np.full(self.n_slots, int(n.max()) + slack, dtype=np.int32)
        total = int(self.capacity.astype(np.int64).sum())
        self.q_all = bits_to_device(ep.q, self.device)
        self.k_all = bits_to_device(ep.k, self.device)
        self.v_all = bits_to_device(ep.v, self.device)
        self.cache_k = torch.full((total, cfg.num_kv_heads, cfg.head_dim), -1, dtype=torch.int16, device=self.device)
        self.cache_v = torch.full_like(self.cache_k, -1)
        self.out_all = torch.zeros_like(self.q_all)
        self.workspace = None
        self.events = []          # ("acquire", id, tokens) | ("pass", BufferedPass) | ("release", id) | ("end", iteration)
        self.removed = []         # per iteration: ids that left
        max_rows = self._trace(max_iterations)
        if use_workspace:
            nbytes = ob.oppo_workspace_bytes(self.desc, self.n_slots, max(1, max_rows))
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.pool = None
        self.cache = None
        self.reset()

    def _trace(self, max_iterations) -> int:
        ep = self.ep
        P, R = ep.prompt_len, ep.resp_len
        sched = ob.oppo_sched_create(self.B, self.delta, self.C)
        pool = ob.oppo_pool_create(self.capacity)
        view = ob.oppo_pool_cache(pool, 0, 0)
        nxt, it_no, max_rows = 0, 0, 0
        streamed = {}
        while (nxt < len(P) or ob.oppo_sched_counts(sched)[0] > 0) and (max_iterations is None or it_no < max_iterations):
            for _ in range(ob.oppo_sched_room(sched)):
                if nxt == len(P):
                    break
                ob.oppo_sched_add(sched, nxt, int(P[nxt]))
                ob.oppo_pool_acquire(pool, nxt, int(P[nxt]) + int(R[nxt]))
                self.events.append(("acquire", nxt, int(P[nxt]) + int(R[nxt])))
                streamed[nxt] = 0
                nxt += 1
            while True:
                kind, ids, kvb, cap = ob.oppo_sched_begin_pass(sched)
                if kind == ob.PASS_NONE:
                    break
                if kind == ob.PASS_PROMPT:
                    q_len = cap.copy()
                else:
                    q_len = np.array([min(int(c), int(R[i]) - streamed[int(i)]) for i, c in zip(ids, cap)], dtype=np.int32)
                cu_q, row_begin = ob.oppo_pool_pack(pool, ids, q_len)
                rows = np.empty(int(cu_q[-1]), dtype=np.int64)
                for i, b, kb, ql in zip(ids, row_begin, kvb, q_len):
                    rows[b:b + ql] = ep.tok_begin[i] + kb + np.arange(ql)
                    view.kv_len[ob.oppo_pool_slot_of(pool, int(i))] += ql     # what oppo_chunk_step will do
                    if kind == ob.PASS_CHUNK:
                        streamed[int(i)] += int(ql)
                fin = np.array([streamed[int(i)] == R[int(i)] for i in ids], dtype=np.uint8)
                ob.oppo_sched_end_pass(sched, ids, q_len, fin)
                trows = torch.from_numpy(rows).to(self.device)
                self.events.append(("pass", BufferedPass(
                    iteration=it_no, kind=kind, ids=ids, kv_before=kvb, q_len=q_len, cu_q=cu_q, rows=trows,
                    q=self.q_all[trows].contiguous(), k=self.k_all[trows].contiguous(), v=self.v_all[trows].contiguous(),
                    out=torch.zeros((len(rows), self.cfg.num_q_heads, self.cfg.head_dim), dtype=torch.int16,
                                    device=self.device))))
                max_rows = max(max_rows, len(rows))
            gone = ob.oppo_sched_end_iteration(sched)
            for i in gone:
                ob.oppo_pool_release(pool, int(i))
                self.events.append(("release", int(i)))
            self.removed.append([int(i) for i in gone])
            self.events.append(("end", it_no))
            it_no += 1
        self.pool_counts = ob.oppo_pool_counts(pool)
        ob.oppo_pool_destroy(pool)
        ob.oppo_sched_destroy(sched)
        return max_rows

    def reset(self) -> None:
        """A fresh pool over the same slabs (the slabs' old contents stay: nothing may read them)."""
        if self.pool is not None:
            ob.oppo_pool_destroy(self.pool)
        self.pool = ob.oppo_pool_create(self.capacity)
        self.cache = ob.oppo_pool_cache(self.pool, self.cache_k, self.cache_v)

    def passes(self) -> List[BufferedPass]:
        return [e[1] for e in self.events if e[0] == "pass"]

    def run(self, stream=None, upto_iteration: Optional[int] = None) -> None:
        """Replays the run from a fresh pool (see reset): every pass is one oppo_chunk_step.
        upto_iteration = k stops after iteration k's sequences have left."""
        for e in self.events:
            if e[0] == "acquire":
                ob.oppo_pool_acquire(self.pool, e[1], e[2])
            elif e[0] == "release":
                ob.oppo_pool_release(self.pool, e[1])
            elif e[0] == "pass":
                p = e[1]
                ob.oppo_chunk_step(self.desc, self.cache, p.cu_q, p.q, p.k, p.v, p.out, self.workspace, stream)
            elif e[0] == "end" and upto_iteration is not None and e[1] >= upto_iteration:
                return

    def scatter_outputs(self) -> torch.Tensor:
        for p in self.passes():
            if len(p.rows):
                self.out_all[p.rows] = p.out
        return self.out_all
