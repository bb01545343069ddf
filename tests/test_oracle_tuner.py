"""Pins of the oracle's chunk-size tuner (Sec. 3.1, periodic search over candidates)."""
import os

import numpy as np

from oracle.tuner import ChunkTunerOracle, run_tuner

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "chunk_tuner_example.txt")


def test_hand_worked_example():
    tables, used = [], None
    for line in open(GOLDEN):
        w = line.split()
        if not w or w[0].startswith("#"):
            continue
        if w[0].startswith("table"):
            tables.append({int(w[i]): float(w[i + 1]) for i in range(1, len(w), 2)})
        elif w[0] == "used":
            used = [int(x) for x in w[1:]]
    got = run_tuner([128, 256, 512], 5, lambda t, c: tables[0 if t < 5 else 1][c], len(used))
    assert got == used


def test_exploits_the_argmin_of_the_windows_trials():
    rng = np.random.default_rng(2)
    for trial in range(50):
        k = int(rng.integers(1, 6))
        cands = [int(x) for x in rng.choice(np.arange(1, 40) * 32, size=k, replace=False)]
        period = int(rng.integers(1, 12))
        cost = rng.random((200, k)) + 0.1                      # cost[t][j]: step t with candidate j
        used = run_tuner(cands, period, lambda t, c: cost[t][cands.index(c)], 200)
        ntr = min(k, period)
        for t, c in enumerate(used):
            start, off = (t // period) * period, t % period
            if off < ntr:
                assert c == cands[off]                         # trials in the order given
            else:
                assert c == cands[int(np.argmin(cost[start:start + ntr, :ntr].diagonal()))]


def test_single_candidate_and_missing_reports():
    assert run_tuner([256], 50, lambda t, c: 1.0, 120) == [256] * 120
    tuner = ChunkTunerOracle([64, 128], 4)
    tuner.report(1, 0.5)                                        # only the second trial was timed
    assert [tuner.chunk_for(t) for t in range(4)] == [64, 128, 128, 128]
    assert [tuner.chunk_for(t) for t in range(4, 8)] == [64, 128, 64, 64]   # nothing reported yet: first candidate
