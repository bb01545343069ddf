"""Host logic of inter-step overlap: the library's Alg. 1 buffer against the oracle's
simulation (exact traces), and the slot pool's bookkeeping.  No GPU."""
import numpy as np
import pytest

from oracle.deferral import simulate
from paper_2509_25762_amd import binding as ob


@pytest.fixture(scope="module")
def lib():
    return ob.load()


def run_library_buffer(P, R, B, delta, C):
    """Drives the library's state machine over the dataset like Alg. 1; the 'actor' knows
    the final response lengths.  Returns the same trace structure the oracle gives."""
    s = ob.oppo_sched_create(B, delta, C)
    nxt, streamed, trace = 0, {}, []
    while nxt < len(P) or ob.oppo_sched_counts(s)[0] > 0:
        it = {"added": [], "passes": [], "removed": [], "carried": None}
        for _ in range(ob.oppo_sched_room(s)):
            if nxt == len(P):
                break
            ob.oppo_sched_add(s, nxt, int(P[nxt]))
            streamed[nxt] = 0
            it["added"].append(nxt)
            nxt += 1
        while True:
            kind, ids, kvb, cap = ob.oppo_sched_begin_pass(s)
            if kind == ob.PASS_NONE:
                break
            if kind == ob.PASS_PROMPT:
                q = cap.copy()
            else:
                q = np.array([min(int(c), int(R[i]) - streamed[int(i)]) for i, c in zip(ids, cap)], dtype=np.int32)
                for i, n in zip(ids, q):
                    streamed[int(i)] += int(n)
            fin = np.array([streamed[int(i)] == R[int(i)] for i in ids], dtype=np.uint8)
            ob.oppo_sched_end_pass(s, ids, q, fin)
            it["passes"].append(("prompt" if kind == ob.PASS_PROMPT else "chunk",
                                 [(int(i), int(k), int(n)) for i, k, n in zip(ids, kvb, q)]))
        it["removed"] = [int(x) for x in ob.oppo_sched_end_iteration(s)]
        trace.append(it)
    ob.oppo_sched_destroy(s)
    return trace


def test_buffer_matches_the_oracle_trace_for_trace(lib):
    rng = np.random.default_rng(21)
    for trial in range(60):
        B, delta, C = int(rng.integers(1, 9)), int(rng.integers(0, 6)), int(rng.integers(1, 16))
        n = int(rng.integers(1, 60))
        P = rng.integers(1, 20, size=n)
        R = np.where(rng.random(n) < 0.1, 0, (rng.pareto(1.5, size=n) * 10).astype(np.int64) + 1)
        want = simulate(P, R, B, delta, C)
        got = run_library_buffer(P, R, B, delta, C)
        assert len(got) == len(want)
        for g, w in zip(got, want):
            assert g["added"] == w.added and g["removed"] == w.removed
            assert g["passes"] == [(p.kind, p.rows) for p in w.passes]


def test_buffer_rejects_calls_out_of_order(lib):
    s = ob.oppo_sched_create(2, 1, 4)
    with pytest.raises(ob.OppoError):
        ob.oppo_sched_end_pass(s, [], [], [])                      # no pass open
    ob.oppo_sched_add(s, 7, 3)
    with pytest.raises(ob.OppoError):
        ob.oppo_sched_add(s, 7, 3)                                 # duplicate
    with pytest.raises(ob.OppoError):
        ob.oppo_sched_add(s, 8, 0)                                 # empty prompt
    ob.oppo_sched_add(s, 8, 2)
    ob.oppo_sched_add(s, 9, 2)
    with pytest.raises(ob.OppoError) as e:
        ob.oppo_sched_add(s, 10, 2)                                # full
    assert e.value.code == ob.OPPO_ERR_CAPACITY
    kind, ids, kvb, cap = ob.oppo_sched_begin_pass(s)
    assert kind == ob.PASS_PROMPT and ids.tolist() == [7, 8, 9] and cap.tolist() == [3, 2, 2] and kvb.tolist() == [0, 0, 0]
    for bad in ([7, 8], [8, 7, 9]):
        with pytest.raises(ob.OppoError):
            ob.oppo_sched_end_pass(s, bad, [1] * len(bad), [0] * len(bad))
    with pytest.raises(ob.OppoError):
        ob.oppo_sched_end_pass(s, ids, [3, 2, 1], [0, 0, 0])       # a prompt pass takes whole prompts
    with pytest.raises(ob.OppoError):
        ob.oppo_sched_begin_pass(s)                                # still open
    with pytest.raises(ob.OppoError):
        ob.oppo_sched_end_iteration(s)
    ob.oppo_sched_end_pass(s, ids, cap, [0, 0, 0])
    kind, ids, kvb, cap = ob.oppo_sched_begin_pass(s)
    assert kind == ob.PASS_CHUNK and kvb.tolist() == [3, 2, 2] and cap.tolist() == [4, 4, 4]
    with pytest.raises(ob.OppoError):
        ob.oppo_sched_end_pass(s, ids, [5, 4, 4], [0, 0, 0])       # more than C
    with pytest.raises(ob.OppoError):
        ob.oppo_sched_end_pass(s, ids, [3, 4, 4], [0, 0, 0])       # short chunk that does not end the sequence
    ob.oppo_sched_end_pass(s, ids, [3, 4, 0], [1, 0, 1])
    assert ob.oppo_sched_counts(s) == (3, 2, 3)
    kind, ids, _, _ = ob.oppo_sched_begin_pass(s)
    assert kind == ob.PASS_NONE and len(ids) == 0                  # B = 2 have finished; nothing is opened
    assert ob.oppo_sched_end_iteration(s).tolist() == [7, 9]
    assert ob.oppo_sched_counts(s) == (1, 0, 3)
    ob.oppo_sched_set_delta(s, 0)                                  # Buffer.set_capacity
    assert ob.oppo_sched_room(s) == 1
    ob.oppo_sched_destroy(s)


def test_slot_pool_bookkeeping(lib):
    pool = ob.oppo_pool_create([10, 5, 20, 5])
    assert ob.oppo_pool_acquire(pool, 100, 4) == 1                 # best fit, lowest index among equals
    assert ob.oppo_pool_acquire(pool, 101, 4) == 3
    assert ob.oppo_pool_acquire(pool, 102, 11) == 2
    with pytest.raises(ob.OppoError) as e:
        ob.oppo_pool_acquire(pool, 103, 11)                        # only the 10-token slot is free
    assert e.value.code == ob.OPPO_ERR_CAPACITY
    with pytest.raises(ob.OppoError):
        ob.oppo_pool_acquire(pool, 100, 1)                         # already owns a slot
    cache = ob.oppo_pool_cache(pool, 0, 0)
    assert cache.batch == 4 and cache.slot_begin.tolist() == [0, 10, 15, 35, 40] and cache.kv_len.tolist() == [0, 0, 0, 0]
    cu_q, row_begin = ob.oppo_pool_pack(pool, [102, 100], [7, 5])  # rows are packed in slot order
    assert cu_q.tolist() == [0, 0, 5, 12, 12] and row_begin.tolist() == [5, 0]
    with pytest.raises(ob.OppoError) as e:
        ob.oppo_pool_pack(pool, [100], [6])                        # 6 tokens into a 5-token slot
    assert e.value.code == ob.OPPO_ERR_CAPACITY
    for bad_ids, bad_len in (([100, 100], [1, 1]), ([555], [1]), ([100], [-1])):
        with pytest.raises(ob.OppoError):
            ob.oppo_pool_pack(pool, bad_ids, bad_len)
    cache.kv_len[1] = 5                                            # as oppo_chunk_step would after 5 rows
    with pytest.raises(ob.OppoError):
        ob.oppo_pool_pack(pool, [100], [1])                        # the slot is full now
    ob.oppo_pool_release(pool, 100)
    assert cache.kv_len[1] == 0                                    # a released slot is empty
    with pytest.raises(ob.OppoError):
        ob.oppo_pool_release(pool, 100)
    with pytest.raises(ob.OppoError):
        ob.oppo_pool_slot_of(pool, 100)
    assert ob.oppo_pool_acquire(pool, 104, 5) == 1 and ob.oppo_pool_slot_of(pool, 104) == 1
    assert ob.oppo_pool_counts(pool) == (4, 3, 4, 1)               # one acquisition reused a slot
    ob.oppo_pool_destroy(pool)


def test_pool_never_gives_one_slot_to_two_live_sequences(lib):
    rng = np.random.default_rng(4)
    cap = rng.integers(1, 50, size=12)
    pool = ob.oppo_pool_create(cap)
    live = {}
    for step in range(2000):
        if live and rng.random() < 0.45:
            sid = int(rng.choice(list(live)))
            ob.oppo_pool_release(pool, sid)
            del live[sid]
        else:
            need = int(rng.integers(0, 55))
            free = [s for s in range(12) if s not in live.values()]
            fits = [s for s in free if cap[s] >= need]
            try:
                slot = ob.oppo_pool_acquire(pool, 10_000 + step, need)
            except ob.OppoError as e:
                assert e.code == ob.OPPO_ERR_CAPACITY and not fits
                continue
            assert slot in fits and cap[slot] == min(cap[s] for s in fits) and slot == min(s for s in fits if cap[s] == cap[slot])
            live[10_000 + step] = slot
        assert len(set(live.values())) == len(live) == ob.oppo_pool_counts(pool)[1]
    ob.oppo_pool_destroy(pool)


def test_chunk_tuner_matches_the_oracle(lib):
    from oracle.tuner import run_tuner
    rng = np.random.default_rng(8)
    for trial in range(40):
        k = int(rng.integers(1, 6))
        cands = [int(x) for x in rng.choice(np.arange(1, 40) * 32, size=k, replace=False)]
        period = int(rng.integers(1, 12))
        n = 150
        cost = np.round(rng.random((n, k)) * 4) / 4 + 0.25          # coarse values: ties do occur
        want = run_tuner(cands, period, lambda t, c: cost[t][cands.index(c)], n)
        tuner = ob.oppo_tuner_create(cands, period)
        got = []
        for t in range(n):
            c = ob.oppo_tuner_chunk(tuner, t)
            got.append(c)
            ob.oppo_tuner_report(tuner, t, float(cost[t][cands.index(c)]))
        ob.oppo_tuner_destroy(tuner)
        assert got == want


def test_chunk_tuner_rejects_bad_arguments(lib):
    for cands, period in (([], 5), ([128, 0], 5), ([128], 0)):
        with pytest.raises(ob.OppoError):
            ob.oppo_tuner_create(cands, period)
    tuner = ob.oppo_tuner_create([64, 128], 4)
    with pytest.raises(ob.OppoError):
        ob.oppo_tuner_chunk(tuner, -1)
    with pytest.raises(ob.OppoError):
        ob.oppo_tuner_report(tuner, 0, -1.0)
    with pytest.raises(ob.OppoError):
        ob.oppo_tuner_report(tuner, 0, float("nan"))
    ob.oppo_tuner_report(tuner, 1, 0.5)                             # only the second trial was timed
    assert [ob.oppo_tuner_chunk(tuner, t) for t in range(8)] == [64, 128, 128, 128, 64, 128, 64, 64]
    ob.oppo_tuner_destroy(tuner)


def test_overlap_timeline_matches_the_oracle(lib):
    from oracle.overlap import timeline
    rng = np.random.default_rng(2024)
    for trial in range(200):
        n = int(rng.integers(0, 12))
        gen = rng.uniform(0.0, 3.0, n) * (rng.random(n) > 0.1)
        score = rng.uniform(0.0, 3.0, n) * (rng.random(n) > 0.1)
        start, end, summ = ob.oppo_overlap_timeline(gen, score)
        want = timeline(gen.tolist(), score.tolist())
        # same additions in the same order on both sides except the prefix sums of gen
        assert np.allclose(start, want["start"], rtol=1e-13, atol=1e-13)
        assert np.allclose(end, want["end"], rtol=1e-13, atol=1e-13)
        for key in ("gen_end", "step_end", "exposed"):
            assert summ[key] == pytest.approx(want[key], rel=1e-13, abs=1e-13)


def test_overlap_timeline_rejects_bad_arguments(lib):
    import ctypes
    summary = (ctypes.c_double * 3)()
    one = (ctypes.c_double * 1)(1.0)
    neg = (ctypes.c_double * 1)(-1.0)
    nan = (ctypes.c_double * 1)(float("nan"))
    f = lib.oppo_overlap_timeline
    assert f(-1, one, one, None, None, summary) == ob.OPPO_ERR_INVALID
    assert f(1, None, one, None, None, summary) == ob.OPPO_ERR_INVALID
    assert f(1, one, one, None, None, None) == ob.OPPO_ERR_INVALID
    assert f(1, neg, one, None, None, summary) == ob.OPPO_ERR_INVALID
    assert f(1, one, nan, None, None, summary) == ob.OPPO_ERR_INVALID
    assert "chunk 0" in ob.oppo_last_error()
    assert f(1, one, one, None, None, summary) == ob.OPPO_OK and list(summary) == [1.0, 2.0, 1.0]
    assert f(0, None, None, None, None, summary) == ob.OPPO_OK and list(summary) == [0.0, 0.0, 0.0]
