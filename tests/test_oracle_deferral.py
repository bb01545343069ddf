"""Pins of the oracle's model of Alg. 1's buffer (B + Delta sequences, inter-step overlap)."""
import os

import numpy as np

from oracle.deferral import simulate, dense_descriptor
from oracle.schedule import chunk_schedule, num_steps

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg1_buffer_example.txt")


def _read_golden():
    P, R, its = [], [], []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = line.split()
        if w[0] == "seq":
            P.append(int(w[2])), R.append(int(w[3]))
        elif w[0] == "iteration":
            its.append({"added": [], "passes": [], "removed": [], "carried": []})
        elif w[0] in ("added", "removed", "carried"):
            its[-1][w[0]] = [int(x) for x in w[1:]]
        elif w[0] == "pass":
            rows = [tuple(int(x) for x in part.split()) for part in line.split(":")[1].split(";")]
            its[-1]["passes"].append((w[1], rows))
    return P, R, its


def test_hand_worked_trace_of_alg1():
    P, R, want = _read_golden()
    got = simulate(P, R, B=2, delta=1, C=2)
    assert len(got) == len(want)
    for g, w in zip(got, want):
        assert g.added == w["added"] and g.removed == w["removed"] and g.carried == w["carried"]
        assert [(p.kind, p.rows) for p in g.passes] == w["passes"]


def test_without_overcommit_it_is_the_plain_streaming_schedule():
    """Delta = 0: every iteration is a batch of B sequences streamed to the end, i.e. the
    passes t = 0.. of the intra-step schedule (Sec. 3.1), preceded by the prompts."""
    rng = np.random.default_rng(5)
    for trial in range(20):
        B, C = int(rng.integers(1, 6)), int(rng.integers(1, 9))
        n = B * int(rng.integers(1, 4))
        P = rng.integers(1, 10, size=n)
        R = rng.integers(1, 30, size=n)
        its = simulate(P, R, B, 0, C)
        assert len(its) == n // B
        for k, it in enumerate(its):
            ids = list(range(k * B, (k + 1) * B))
            assert it.added == ids and sorted(it.removed) == ids and it.carried == []
            assert it.passes[0].kind == "prompt" and it.passes[0].rows == [(i, 0, int(P[i])) for i in ids]
            chunks = it.passes[1:]
            assert len(chunks) == num_steps(R[ids], C)
            for t, p in enumerate(chunks):
                kvb, ql, _ = chunk_schedule(P[ids], R[ids], C, t)
                assert p.rows == [(ids[j], int(kvb[j]), int(ql[j])) for j in range(B) if ql[j] > 0]


def test_invariants_of_the_buffer():
    rng = np.random.default_rng(9)
    for trial in range(40):
        B, delta, C = int(rng.integers(1, 7)), int(rng.integers(0, 5)), int(rng.integers(1, 12))
        n = int(rng.integers(1, 40))
        P = rng.integers(1, 12, size=n)
        R = np.where(rng.random(n) < 0.1, 0, rng.integers(1, 60, size=n))   # long tail and a few empty responses
        its = simulate(P, R, B, delta, C)
        in_buffer, seen_prompt, streamed, removed_at, finished_at = [], set(), {}, {}, {}
        clock = 0
        for it in its:
            in_buffer += it.added
            assert len(in_buffer) <= B + delta                                  # capacity
            assert it.added == list(range(len(seen_prompt), len(seen_prompt) + len(it.added)))   # dataset order
            for p in it.passes:
                clock += 1
                ids = [r[0] for r in p.rows]
                assert len(set(ids)) == len(ids) and set(ids) <= set(in_buffer)
                assert ids == [i for i in in_buffer if i in set(ids)]           # buffer (FIFO) order
                if p.kind == "prompt":
                    assert ids == it.added
                    for i, kvb, q in p.rows:
                        assert kvb == 0 and q == P[i] and i not in seen_prompt
                        seen_prompt.add(i)
                        streamed[i] = 0
                        if R[i] == 0:
                            finished_at[i] = clock
                else:
                    # every unfinished sequence of the buffer is served: nobody starves
                    assert ids == [i for i in in_buffer if streamed[i] < R[i]]
                    for i, kvb, q in p.rows:
                        assert kvb == P[i] + streamed[i]                        # nothing recomputed, nothing skipped
                        assert 1 <= q <= C and (q == C or streamed[i] + q == R[i])
                        streamed[i] += q
                        if streamed[i] == R[i]:
                            finished_at[i] = clock
            assert len(it.removed) <= B and len(set(it.removed)) == len(it.removed)
            for i in it.removed:
                assert streamed[i] == R[i] and i in in_buffer and i not in removed_at
                removed_at[i] = it.index
            assert [finished_at[i] for i in it.removed] == sorted(finished_at[i] for i in it.removed)
            # the removed ones are the earliest finishers among those finished and present
            waiting = [i for i in in_buffer if i in finished_at and i not in it.removed]
            if waiting:
                assert len(it.removed) == B
                assert max(finished_at[i] for i in it.removed) <= min(finished_at[i] for i in waiting)
            in_buffer = [i for i in in_buffer if i not in set(it.removed)]
            assert it.carried == in_buffer
        assert sorted(removed_at) == list(range(n)) and in_buffer == []         # everybody leaves exactly once


def test_dense_descriptor():
    P, R, _ = _read_golden()
    its = simulate(P, R, 2, 1, 2)
    p = its[1].passes[1]                       # chunk pass with ids 0, 3, 4
    kvb, ql, cu = dense_descriptor(p, {0: 2, 3: 0, 4: 1}, 4)
    assert kvb.tolist() == [1, 1, 5, 0] and ql.tolist() == [2, 2, 2, 0] and cu.tolist() == [0, 2, 4, 6, 6]
