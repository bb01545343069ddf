"""The buffer of Alg. 1 with inter-step overlap, as a plain simulation (test oracle).

Sec. 3.2 / Alg. 1: the buffer holds B + Delta sequences.  Every training
iteration first fills it up with new sequences (stage 1), then streams chunks of
up to C tokens to every unfinished sequence, pass after pass, until B sequences
have finished (stage 2; the scorer prefills each chunk on top of what it already
holds, Sec. 3.1), then removes the first B finished sequences (stage 3).  The
unfinished ones stay, with everything the scorer has cached for them, and go on
in the next iteration.

With final response lengths R_i known in advance the whole run is determined.
This module lists, pass by pass, which sequence contributes how many new rows on
top of how many cached tokens - the ragged descriptors the scorer's attention is
called with - and which sequences enter and leave the buffer when.

Readings of the algorithm where it leaves a choice:
  * The buffer is first-in first-out: `finished` lists sequences in the order in
    which they finished, and within one pass in buffer order; "the first B
    completed" are the first B of that list.
  * A sequence that finished but was not among the B removed ones stays in the
    buffer as finished; it counts towards the B of the next iteration and is
    first in line there.  (The listing re-initialises `finished` per iteration;
    without this reading such a sequence could never leave the buffer.)
  * A new sequence's prompt is prefilled by the scorer in a pass of its own kind
    when the sequence enters the buffer (stage 1): q_len = P_i on an empty cache,
    every other sequence sits that pass out.
  * The generation loop also ends when nothing is unfinished (as in the listing),
    and the run ends when the dataset is exhausted and the buffer is empty.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np


class Pass:
    """One call of the scorer: (sequence id, kv_before, q_len) for every sequence
    that has rows in it.  `kind` is "prompt" (stage 1) or "chunk" (stage 2)."""

    def __init__(self, kind: str, iteration: int, rows: List[Tuple[int, int, int]]):
        self.kind, self.iteration, self.rows = kind, iteration, rows

    def __repr__(self) -> str:
        return f"Pass({self.kind}, it={self.iteration}, {self.rows})"


class Iteration:
    def __init__(self, index: int):
        self.index = index
        self.added: List[int] = []        # ids that entered the buffer in stage 1, in order
        self.passes: List[Pass] = []      # the scorer's passes of this iteration, in order
        self.removed: List[int] = []      # the PPO batch (stage 3), in finishing order
        self.carried: List[int] = []      # what stays in the buffer afterwards, in buffer order


def simulate(prompt_len: Sequence[int], resp_len: Sequence[int], B: int, delta: int, C: int,
             max_iterations: int = 10 ** 9) -> List[Iteration]:
    """Runs Alg. 1 over the dataset (sequence i = prompt_len[i], resp_len[i], taken
    in index order) until it is exhausted and the buffer is empty, or for
    `max_iterations` iterations."""
    assert B >= 1 and delta >= 0 and C >= 1
    P = [int(x) for x in prompt_len]
    R = [int(x) for x in resp_len]
    assert len(P) == len(R) and all(p >= 1 for p in P) and all(r >= 0 for r in R)
    nxt = 0                               # next dataset index
    buffer: List[int] = []                # ids in FIFO order
    done: Dict[int, int] = {}             # response tokens streamed so far
    finished_order: List[int] = []        # finished and still in the buffer, in finishing order
    out: List[Iteration] = []
    while len(out) < max_iterations and (nxt < len(P) or buffer):
        it = Iteration(len(out))
        # stage 1: fill the buffer to capacity
        while len(buffer) < B + delta and nxt < len(P):
            buffer.append(nxt)
            done[nxt] = 0
            it.added.append(nxt)
            nxt += 1
        if it.added:
            it.passes.append(Pass("prompt", it.index, [(i, 0, P[i]) for i in it.added]))
            for i in it.added:            # an empty response is finished on arrival
                if R[i] == 0:
                    finished_order.append(i)
        # stage 2: generation with intra-step overlap
        while len(finished_order) < B:
            active = [i for i in buffer if done[i] < R[i]]
            if not active:
                break
            rows = []
            for i in active:
                q = min(C, R[i] - done[i])
                rows.append((i, P[i] + done[i], q))
            it.passes.append(Pass("chunk", it.index, rows))
            for i, _, q in rows:
                done[i] += q
                if done[i] == R[i]:
                    finished_order.append(i)
        # stage 3: the first B finished sequences leave
        it.removed = finished_order[:B]
        finished_order = finished_order[B:]
        gone = set(it.removed)
        buffer = [i for i in buffer if i not in gone]
        it.carried = list(buffer)
        out.append(it)
    return out


def dense_descriptor(p: Pass, slot_of: Dict[int, int], n_slots: int):
    """The pass as the library's per-slot arrays: (kv_before[n_slots], q_len[n_slots],
    cu_q[n_slots+1]); slots without rows in this pass have q_len 0."""
    kv_before = np.zeros(n_slots, dtype=np.int64)
    q_len = np.zeros(n_slots, dtype=np.int64)
    for i, kvb, q in p.rows:
        s = slot_of[i]
        assert q_len[s] == 0, "two sequences of one pass in one slot"
        kv_before[s], q_len[s] = kvb, q
    cu_q = np.zeros(n_slots + 1, dtype=np.int64)
    np.cumsum(q_len, out=cu_q[1:])
    return kv_before, q_len, cu_q
