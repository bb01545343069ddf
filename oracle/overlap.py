"""Timeline of intra-step overlap: the actor decodes chunk k while the scorer
prefills chunk k-1 (test oracle).

Sec. 3.1: the actor's generation is cut into chunks that are streamed to the
scorer; scoring proceeds while generation goes on, and at the end of the step
the scorer finishes the prefill of the last chunk.  What the technique buys is
the scoring time that is hidden behind generation; what remains exposed is the
time between the end of generation and the end of the last chunk's scoring.

The model, written out as its definition:
  * the actor decodes its chunks back to back from time 0; chunk k is complete
    at ready[k] = gen[0] + ... + gen[k];
  * the scorer is one server that takes the chunks in order, one at a time;
    it starts chunk k when chunk k is complete and chunk k-1 has been scored;
  * without streaming (the baseline the paper compares with) all scoring
    happens after generation: the step ends at sum(gen) + score_once.
Readings: neither side slows the other down (separate GPUs; the colocated case
is a measurement, not part of this model), and a chunk is handed over whole.
"""
from __future__ import annotations

from typing import Dict, List, Sequence


def timeline(gen: Sequence[float], score: Sequence[float]) -> Dict[str, object]:
    """gen[k] / score[k]: time the actor needs to decode, the scorer to prefill, chunk k."""
    assert len(gen) == len(score)
    assert all(g >= 0 for g in gen) and all(s >= 0 for s in score)
    start: List[float] = []
    end: List[float] = []
    for k in range(len(gen)):
        ready = float(sum(gen[: k + 1]))
        free = end[k - 1] if k else 0.0
        start.append(max(ready, free))
        end.append(start[k] + float(score[k]))
    gen_end = float(sum(gen))
    step_end = end[-1] if end else 0.0
    return {"start": start, "end": end, "gen_end": gen_end, "step_end": max(step_end, gen_end),
            "exposed": max(step_end - gen_end, 0.0)}


def sequential_step(gen: Sequence[float], score_once: float) -> float:
    """Step time without streaming: generation, then one prefill of everything."""
    return float(sum(gen)) + float(score_once)
