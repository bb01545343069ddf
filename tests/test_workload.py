"""Generator tests (CPU): seeds reproduce, bounds hold, stragglers forced."""
import numpy as np
import pytest

from paper_2509_25762_amd.workload import (CONFIGS, build_episode, draw_lengths, draw_tensor_bits,
                                            f32_to_bf16_bits, step_work)


def test_lengths_reproduce_and_respect_bounds():
    for cfg in CONFIGS.values():
        P, R = draw_lengths(cfg)
        P2, R2 = draw_lengths(cfg)
        assert np.array_equal(P, P2) and np.array_equal(R, R2)
        assert P.shape == (cfg.batch,) and R.shape == (cfg.batch,)
        if cfg.prompt[0] == "uniform":
            assert P.min() >= cfg.prompt[1] and P.max() <= cfg.prompt[2]
        else:
            assert np.all(P == cfg.prompt[1])
        if cfg.response[0] == "lognormal":
            assert R.min() >= cfg.response[3] and R.max() <= cfg.response[4]
        else:
            assert np.all(R == cfg.response[1])


def test_long_tail_config_has_forced_stragglers():
    cfg = CONFIGS[4]
    _, R = draw_lengths(cfg)
    assert int(np.sum(R == 8192)) >= 2  # ceil(0.05 * 32) = 2 forced


def test_lognormal_median_is_plausible():
    cfg = CONFIGS[3]
    _, R = draw_lengths(cfg)
    med = float(np.median(R))
    assert 150 <= med <= 420  # median 256, sigma 1.0, 256 draws


def test_bf16_rounding_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, 1.005, -2.5, 0.0], dtype=np.float32)
    # 1.00390625 = 1 + 2^-8 is a tie between 0x3F80 and 0x3F81 -> even (0x3F80)
    # 1.01171875 = 1 + 3*2^-8 is a tie between 0x3F81 and 0x3F82 -> even (0x3F82)
    got = f32_to_bf16_bits(x)
    assert got.tolist() == [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xC020, 0x0000]


def test_tensor_streams_are_independent_and_reproducible():
    a = draw_tensor_bits(5, 0, 0, (4, 2, 8))
    assert np.array_equal(a, draw_tensor_bits(5, 0, 0, (4, 2, 8)))
    assert not np.array_equal(a, draw_tensor_bits(5, 0, 1, (4, 2, 8)))
    assert not np.array_equal(a, draw_tensor_bits(5, 1, 0, (4, 2, 8)))


def test_episode_packing_tiny():
    cfg = CONFIGS[1]
    ep = build_episode(cfg, threads=2)
    assert ep.tok_begin[-1] == int((ep.prompt_len.astype(np.int64) + ep.resp_len).sum())
    assert ep.q.shape == (ep.tok_begin[-1], 4, 64) and ep.k.shape == (ep.tok_begin[-1], 4, 64)
    i = 2
    lo, hi = int(ep.tok_begin[i]), int(ep.tok_begin[i + 1])
    assert np.array_equal(ep.v[lo:hi], draw_tensor_bits(cfg.seed, i, 2, (hi - lo, 4, 64)))
    assert ep.num_steps == 4


def test_step_work_counts_visible_pairs():
    cfg = CONFIGS[1]
    w = step_work(cfg, np.array([10, 0, 7]), np.array([2, 3, 0]))
    # pairs: seq0 rows see 11 and 12 keys; seq1 rows see 1, 2, 3; seq2 inactive
    assert w["flops"] == 4.0 * 64 * 4 * (11 + 12 + 1 + 2 + 3)
    assert w["kv_read_bytes"] == (12 + 3) * 4 * 64 * 2 * 2
    assert w["rows"] == 5 and w["active"] == 2


def test_timing_model_of_the_generating_side():
    """The synthetic timing model that stands in for the actor (stated figures, not the method):
    a decode step reads the weights and every live token's K/V once; a chunk is its steps plus one
    hand-off; per-chunk and per-pass bookkeeping agree."""
    from bench import TimingModel, generation_times, pass_generation_time
    m = TimingModel()
    assert m.decode_step_s(0) == pytest.approx(m.decode_step_overhead_s + m.weight_bytes / m.decode_bytes_per_s)
    assert m.decode_step_s(1000) - m.decode_step_s(0) == pytest.approx(1000 * m.kv_bytes_per_token / m.decode_bytes_per_s)
    assert m.dense_s(10) == pytest.approx(10 * m.dense_flops_per_token / m.dense_flops_per_s)
    P = np.array([5, 9, 2], dtype=np.int64)
    R = np.array([7, 3, 0], dtype=np.int64)
    # by hand: steps j = 0..6; live tokens P_i + j summed over sequences with R_i > j
    live = [(5 + j) + ((9 + j) if j < 3 else 0) for j in range(7)]
    step = [m.decode_step_s(x) for x in live]
    g = generation_times(P, R, 4, m)
    assert len(g) == 2
    assert g[0] == pytest.approx(m.handoff_s + sum(step[:4]))
    assert g[1] == pytest.approx(m.handoff_s + sum(step[4:]))
    # the same chunks as passes of a schedule: (kv_before, q_len) of the sequences with rows
    assert pass_generation_time([5, 9], [4, 3], m) == pytest.approx(g[0])
    assert pass_generation_time([9], [3], m) == pytest.approx(g[1])
    assert pass_generation_time([], [], m) == pytest.approx(m.handoff_s)
    # smaller chunks: same decode steps, more hand-offs
    assert sum(generation_times(P, R, 1, m)) == pytest.approx(sum(g) + 5 * m.handoff_s)
