"""GPU parity of inter-step overlap (Sec. 3.2, Alg. 1): B + Delta cache slots, sequences
that finish leave, unfinished ones keep their cached state across iterations, new ones
take over released slots.  Every pass is one oppo_chunk_step over all slots.

The oracle side: every output row equals one-shot causal attention over the row's own
sequence (float64), whatever slot the sequence lived in and whoever lived there before;
the passes are those of the oracle's simulation of Alg. 1; mid-run, the slabs of the
sequences in the buffer hold exactly their tokens so far.
"""
import numpy as np
import pytest

from oracle import bf16_bits_to_f64, full_prefill, simulate_alg1_buffer
from paper_2509_25762_amd.workload import Config, build_episode

pytestmark = pytest.mark.gpu

MAX_ABS = 2e-2
MEAN_ABS = 2e-3

CASES = [
    # long-tailed responses, a few empty ones; chunk not a multiple of the 64-token query tile
    dict(cfg=Config(0, "deferral-gqa", 777, 14, 8, 2, 128, 48, ("uniform", 20, 90), ("lognormal", 90, 1.0, 1, 700)),
         B=4, delta=2, empty=(3, 9)),
    dict(cfg=Config(0, "deferral-mha-d64", 778, 11, 4, 4, 64, 64, ("uniform", 1, 130), ("lognormal", 150, 0.9, 1, 900)),
         B=3, delta=3, empty=()),
    dict(cfg=Config(0, "deferral-none", 779, 6, 4, 2, 128, 32, ("uniform", 10, 40), ("lognormal", 60, 0.7, 1, 300)),
         B=3, delta=0, empty=()),
]


@pytest.fixture(scope="module")
def gpu():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2509_25762_amd import binding, episode
    binding.load()
    return binding, episode, torch


def make_episode(case):
    cfg = case["cfg"]
    from paper_2509_25762_amd.workload import draw_lengths
    P, R = draw_lengths(cfg)
    R = R.copy()
    for i in case["empty"]:
        R[i] = 0
    return build_episode(cfg, threads=4, lengths=(P, R))


@pytest.mark.parametrize("case", CASES, ids=[c["cfg"].name for c in CASES])
def test_buffered_run_matches_oracle(gpu, case):
    ob, episode, torch = gpu
    ep = make_episode(case)
    cfg, B, delta = ep.cfg, case["B"], case["delta"]
    print(f"case {cfg.name}: B={B} delta={delta} C={cfg.chunk} P={ep.prompt_len.tolist()} R={ep.resp_len.tolist()}", flush=True)
    want = simulate_alg1_buffer(ep.prompt_len, ep.resp_len, B, delta, cfg.chunk)
    run = episode.BufferedRun(ep, B, delta, cfg.chunk)
    # the driver's passes are the oracle's
    got_passes = [(p.iteration, "prompt" if p.kind == ob.PASS_PROMPT else "chunk",
                   [(int(i), int(k), int(q)) for i, k, q in zip(p.ids, p.kv_before, p.q_len)]) for p in run.passes()]
    assert got_passes == [(it.index, p.kind, p.rows) for it in want for p in it.passes]
    assert run.removed == [it.removed for it in want]
    if delta:
        assert any(it.carried for it in want), "the case must carry sequences over"
        assert run.pool_counts[3] > 0, "the case must reuse slots"
    run.run()
    torch.cuda.synchronize()
    out = run.scatter_outputs().cpu().numpy().view(np.uint16)
    worst, total, count = 0.0, 0.0, 0
    for i in range(cfg.batch):
        lo, hi = int(ep.tok_begin[i]), int(ep.tok_begin[i + 1])
        ref = full_prefill(bf16_bits_to_f64(ep.q[lo:hi]), bf16_bits_to_f64(ep.k[lo:hi]), bf16_bits_to_f64(ep.v[lo:hi]),
                           cfg.softmax_scale)
        err = np.abs(bf16_bits_to_f64(out[lo:hi]) - ref)
        assert np.isfinite(err).all()
        worst, total, count = max(worst, float(err.max())), total + float(err.sum()), count + err.size
    assert worst <= MAX_ABS and total / count <= MEAN_ABS, (worst, total / count)
    assert ob.oppo_pool_counts(run.pool)[1] == 0                   # everybody has left


def test_carried_sequences_keep_their_cache(gpu):
    """Stop after an iteration that carries sequences over: their slabs hold exactly their
    tokens so far (bit for bit), lengths are prompt + streamed, released slots are empty."""
    ob, episode, torch = gpu
    case = CASES[0]
    ep = make_episode(case)
    cfg, B, delta = ep.cfg, case["B"], case["delta"]
    want = simulate_alg1_buffer(ep.prompt_len, ep.resp_len, B, delta, cfg.chunk)
    k_it = next(it.index for it in want if it.carried and it.index >= 1)
    print(f"stopping after iteration {k_it}: carried {want[k_it].carried}", flush=True)
    run = episode.BufferedRun(ep, B, delta, cfg.chunk)
    run.run(upto_iteration=k_it)
    torch.cuda.synchronize()
    streamed = {}
    for it in want[: k_it + 1]:
        for p in it.passes:
            if p.kind == "chunk":
                for i, _, q in p.rows:
                    streamed[i] = streamed.get(i, 0) + q
    ck = run.cache_k.cpu().numpy().view(np.uint16)
    cv = run.cache_v.cpu().numpy().view(np.uint16)
    live_slots = set()
    for i in want[k_it].carried:
        slot = ob.oppo_pool_slot_of(run.pool, i)
        live_slots.add(slot)
        n = int(ep.prompt_len[i]) + streamed.get(i, 0)
        assert run.cache.kv_len[slot] == n
        b, lo = int(run.cache.slot_begin[slot]), int(ep.tok_begin[i])
        assert np.array_equal(ck[b:b + n], ep.k[lo:lo + n]) and np.array_equal(cv[b:b + n], ep.v[lo:lo + n])
    assert len(live_slots) == len(want[k_it].carried) == ob.oppo_pool_counts(run.pool)[1]
    for slot in range(run.n_slots):
        if slot not in live_slots:
            assert run.cache.kv_len[slot] == 0
