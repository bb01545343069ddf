"""The periodic chunk-size search of intra-step overlap (test oracle).

Sec. 3.1, "Dynamic Control on Intra-step Overlap": the best chunk size depends on
model and workload, the trade-off is monotonic on either side of the optimum and
training runs for many steps, so every `period` training steps a few candidate
chunk sizes are each applied to one step, and the one whose step was fastest is
used for the remaining steps of the window.

Readings where the paper leaves a choice: a window starts with the trials, one
step per candidate in the order given; the choice is made from the step times of
this window's trials only; ties go to the candidate listed first; a step whose
time was never reported counts as infinitely slow; if the window is shorter than
the list of candidates, only the first `period` candidates are tried.
"""
from __future__ import annotations

from typing import Dict, List, Sequence


class ChunkTunerOracle:
    def __init__(self, candidates: Sequence[int], period: int):
        assert len(candidates) >= 1 and all(int(c) >= 1 for c in candidates) and period >= 1
        self.candidates = [int(c) for c in candidates]
        self.period = int(period)
        self.times: Dict[int, float] = {}     # training step -> reported step time

    def _trials(self) -> int:
        return min(len(self.candidates), self.period)

    def chunk_for(self, step: int) -> int:
        """Chunk size to use for training step `step` (0, 1, 2, ...)."""
        assert step >= 0
        start = (step // self.period) * self.period
        k = step - start
        if k < self._trials():
            return self.candidates[k]
        best, best_time = 0, float("inf")
        for j in range(self._trials()):
            t = self.times.get(start + j, float("inf"))
            if t < best_time:
                best, best_time = j, t
        return self.candidates[best]

    def report(self, step: int, seconds: float) -> None:
        assert step >= 0 and seconds >= 0.0
        self.times[step] = float(seconds)


def run_tuner(candidates: Sequence[int], period: int, step_time, n_steps: int) -> List[int]:
    """Chunk sizes the tuner applies over n_steps when step `t` run with chunk C takes
    step_time(t, C) seconds."""
    tuner = ChunkTunerOracle(candidates, period)
    used = []
    for t in range(n_steps):
        c = tuner.chunk_for(t)
        used.append(c)
        tuner.report(t, step_time(t, c))
    return used
