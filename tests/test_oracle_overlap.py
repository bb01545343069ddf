"""Pins of the intra-step overlap timeline (oracle/overlap.py): a hand-worked
golden file, a tick-by-tick simulation on integer durations, and closed forms."""
import os

import numpy as np
import pytest

from oracle.overlap import sequential_step, timeline

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "overlap_timeline_example.txt")


def read_cases():
    cases, cur = [], None
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        if key == "case":
            cur = {"name": vals[0]}
            cases.append(cur)
        else:
            cur[key] = [float(v) for v in vals]
    return cases


@pytest.mark.parametrize("case", read_cases(), ids=lambda c: c["name"])
def test_hand_worked_examples(case):
    t = timeline(case["gen"], case["score"])
    assert t["start"] == case["start"]
    assert t["end"] == case["end"]
    assert t["exposed"] == case["exposed"][0]
    assert t["gen_end"] == sum(case["gen"])


def tick_simulation(gen, score):
    """One time unit per tick: the actor works through its chunks; the scorer works on the
    oldest complete, unscored chunk.  Returns per-chunk (first tick worked on, tick finished)."""
    n = len(gen)
    g_left, s_left = list(gen), list(score)
    start, end = [None] * n, [None] * n
    g_cur = s_cur = 0
    tick = 0
    while s_cur < n:
        # chunks with nothing to decode / score complete at once
        while g_cur < n and g_left[g_cur] == 0:
            g_cur += 1
        while s_cur < n and s_cur < g_cur and s_left[s_cur] == 0:
            if start[s_cur] is None:
                start[s_cur] = tick
            end[s_cur] = tick
            s_cur += 1
        if s_cur >= n:
            break
        scorer_can_work = s_cur < g_cur          # decided before the actor's work of this tick
        if g_cur < n:
            g_left[g_cur] -= 1
        if scorer_can_work:
            if start[s_cur] is None:
                start[s_cur] = tick
            s_left[s_cur] -= 1
            if s_left[s_cur] == 0:
                end[s_cur] = tick + 1
                s_cur += 1
        tick += 1
    return start, end


def test_against_tick_by_tick_simulation():
    rng = np.random.default_rng(31)
    for trial in range(300):
        n = int(rng.integers(1, 8))
        gen = [int(x) for x in rng.integers(0, 7, n)]
        score = [int(x) for x in rng.integers(1, 7, n)]
        t = timeline(gen, score)
        start, end = tick_simulation(gen, score)
        assert t["start"] == [float(x) for x in start], (gen, score)
        assert t["end"] == [float(x) for x in end], (gen, score)


def test_closed_forms():
    rng = np.random.default_rng(7)
    for _ in range(100):
        n = int(rng.integers(1, 10))
        gen = rng.uniform(1.0, 2.0, n)
        # scorer always done before the next chunk arrives: only the last chunk is exposed
        score = np.minimum(rng.uniform(0.1, 1.0, n), np.append(gen[1:], np.inf))
        t = timeline(gen, score)
        assert t["exposed"] == pytest.approx(score[-1])
        # scorer never idle after the first chunk: step = gen[0] + sum(score)
        slow = gen.max() + rng.uniform(0.0, 1.0, n)
        t = timeline(gen, slow)
        assert t["step_end"] == pytest.approx(gen[0] + slow.sum())
        # one chunk = no streaming = the sequential baseline
        t1 = timeline([gen.sum()], [slow.sum()])
        assert t1["step_end"] == pytest.approx(sequential_step(gen, slow.sum()))


def test_bounds_and_monotonicity():
    rng = np.random.default_rng(8)
    for _ in range(200):
        n = int(rng.integers(1, 10))
        gen, score = rng.uniform(0, 3, n), rng.uniform(0, 3, n)
        t = timeline(gen, score)
        assert t["exposed"] >= score[-1] - 1e-12                      # the last chunk can never be hidden
        assert t["step_end"] <= gen.sum() + score.sum() + 1e-12       # never worse than no overlap at all
        assert t["step_end"] >= max(gen.sum() + score[-1], gen[0] + score.sum()) - 1e-12
        k = int(rng.integers(0, n))
        more = score.copy()
        more[k] += 1.0
        assert timeline(gen, more)["step_end"] >= t["step_end"] - 1e-12
        for a, b in zip(t["start"], t["end"]):
            assert b >= a
        assert all(t["start"][i + 1] >= t["end"][i] for i in range(n - 1))  # one chunk at a time


def test_empty():
    t = timeline([], [])
    assert t["start"] == [] and t["exposed"] == 0.0 and t["step_end"] == 0.0
