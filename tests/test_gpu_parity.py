"""GPU parity: the HIP path, called through the C ABI, against the float64 oracle.

Tolerances (bf16 outputs widened to float64 vs the unrounded oracle):
max abs <= 2e-2 and mean abs <= 2e-3; cache contents and positions bit-exact.
"""
import numpy as np
import pytest

from oracle import attention_row, bf16_bits_to_f64, chunk_schedule, full_prefill, num_steps
from paper_2509_25762_amd.workload import CONFIGS, Config, build_episode

pytestmark = pytest.mark.gpu

MAX_ABS = 2e-2
MEAN_ABS = 2e-3


@pytest.fixture(scope="module")
def gpu():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2509_25762_amd import binding, episode
    binding.load()  # fails loudly if the HIP library is not built
    yield binding, episode, torch
    binding.oppo_set_option(binding.OPT_SPLIT_KV, 0)
    binding.oppo_set_option(binding.OPT_ORDER, 0)


def small_cfg(B, Hq, Hkv, D, C, seed=1234):
    return Config(99, "case", seed, B, Hq, Hkv, D, C, ("fixed", 1), ("fixed", 1))


def oracle_outputs(ep):
    outs = np.empty(ep.q.shape, dtype=np.float64)
    for i in range(ep.cfg.batch):
        lo, hi = int(ep.tok_begin[i]), int(ep.tok_begin[i + 1])
        outs[lo:hi] = full_prefill(bf16_bits_to_f64(ep.q[lo:hi]), bf16_bits_to_f64(ep.k[lo:hi]),
                                   bf16_bits_to_f64(ep.v[lo:hi]), ep.cfg.softmax_scale)
    return outs


def oracle_uniform_chunks(P, R, C):
    steps = [[int(p) for p in P]]
    for t in range(num_steps(R, C)):
        steps.append([int(x) for x in chunk_schedule(P, R, C, t)[1]])
    return steps


def check_outputs(got_bits, ref, what=""):
    got = bf16_bits_to_f64(got_bits)
    err = np.abs(got - ref)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert err.max() <= MAX_ABS, f"{what}: max abs {err.max():.4e} at {np.unravel_index(err.argmax(), err.shape)}"
    assert err.mean() <= MEAN_ABS, f"{what}: mean abs {err.mean():.4e}"
    return err.max(), err.mean()


def check_cache(se, ep, torch):
    """Every slot of the slabs: valid tokens bit-exact, everything else still 0xFFFF."""
    ck = se.cache_k.cpu().numpy().view(np.uint16)
    cv = se.cache_v.cpu().numpy().view(np.uint16)
    want_k = np.full(ck.shape, 0xFFFF, dtype=np.uint16)
    want_v = np.full(cv.shape, 0xFFFF, dtype=np.uint16)
    for i in range(ep.cfg.batch):
        n = int(se.total_done[i])
        b = int(se.slot_begin[i])
        lo = int(ep.tok_begin[i])
        want_k[b:b + n] = ep.k[lo:lo + n]
        want_v[b:b + n] = ep.v[lo:lo + n]
        assert se.cache.kv_len[i] == n
    assert np.array_equal(ck, want_k), "K cache differs"
    assert np.array_equal(cv, want_v), "V cache differs"


def run_and_check(gpu, ep, chunks, ref=None, what=""):
    """Streams the episode twice - with the fused call (oppo_chunk_step) and with
    oppo_kv_append + oppo_chunk_prefill_attn - and checks both against the oracle;
    the two must agree bit for bit, in the outputs and in the cache."""
    binding, episode, torch = gpu
    ref = oracle_outputs(ep) if ref is None else ref
    outs = []
    for fused in (False, True):
        se = episode.StreamedEpisode(ep, chunks)
        se.run(fused=fused)
        torch.cuda.synchronize()
        out = se.scatter_outputs().cpu().numpy().view(np.uint16)
        res = check_outputs(out, ref, f"{what} fused={fused}")
        check_cache(se, ep, torch)
        outs.append(out)
    assert np.array_equal(outs[0], outs[1]), f"{what}: fused and two-call results differ"
    return se, out, res


# --------------------------------------------------------------------------- tiny config, exhaustive

@pytest.fixture(scope="module")
def tiny_ep():
    ep = build_episode(CONFIGS[1], threads=2)
    return ep, oracle_outputs(ep)


def test_tiny_canonical_chunking_all_rows(gpu, tiny_ep):
    ep, ref = tiny_ep
    _, _, (mx, mean) = run_and_check(gpu, ep, oracle_uniform_chunks(ep.prompt_len, ep.resp_len, 32), ref, "tiny C=32")
    print(f"tiny: max abs {mx:.3e} mean abs {mean:.3e}")


@pytest.mark.parametrize("C", [1, 7, 10, 31, 33, 64, 100, 127, 128, 500])
def test_tiny_uniform_chunkings_equal_one_shot(gpu, tiny_ep, C):
    ep, ref = tiny_ep
    run_and_check(gpu, ep, oracle_uniform_chunks(ep.prompt_len, ep.resp_len, C), ref, f"tiny C={C}")


def test_tiny_random_compositions_and_deferral(gpu, tiny_ep):
    ep, ref = tiny_ep
    B = ep.cfg.batch
    rng = np.random.default_rng(5)
    for trial in range(4):
        left = (ep.prompt_len.astype(np.int64) + ep.resp_len).tolist()
        chunks = []
        while any(left):
            step = []
            for i in range(B):
                take = 0 if rng.random() < 0.25 else int(rng.integers(1, 90))
                take = min(take, left[i])
                left[i] -= take
                step.append(take)
            chunks.append(step)
        run_and_check(gpu, ep, chunks, ref, f"tiny composition {trial}")


def test_tiny_gpu_chunked_equals_gpu_full_prefill(gpu, tiny_ep):
    binding, episode, torch = gpu
    ep, ref = tiny_ep
    se, out, _ = run_and_check(gpu, ep, oracle_uniform_chunks(ep.prompt_len, ep.resp_len, 32), ref)
    full = se.full_prefill()
    torch.cuda.synchronize()
    full = full.cpu().numpy().view(np.uint16)
    check_outputs(full, ref, "gpu full prefill")
    d = np.abs(bf16_bits_to_f64(full) - bf16_bits_to_f64(out))
    assert d.max() <= MAX_ABS and d.mean() <= MEAN_ABS
    print(f"bit-identical outputs chunked vs one-shot: {np.mean(full == out) * 100:.2f}%")


def test_first_token_is_its_value_bit_exact(gpu, tiny_ep):
    ep, ref = tiny_ep
    _, out, _ = run_and_check(gpu, ep, oracle_uniform_chunks(ep.prompt_len, ep.resp_len, 32), ref)
    for i in range(ep.cfg.batch):
        lo = int(ep.tok_begin[i])
        for h in range(ep.cfg.num_q_heads):
            assert np.array_equal(out[lo, h], ep.v[lo, h // ep.cfg.group])


# --------------------------------------------------------------------------- shapes, tiles, ragged tails

CASES = [
    # B, Hq, Hkv, D, prompts, responses, C
    ("gqa4_d128", 5, 8, 2, 128, [70, 130, 1, 257, 64], [100, 5, 300, 64, 129], 48),
    ("gqa8_d128", 3, 16, 2, 128, [33, 200, 5], [90, 17, 260], 64),
    ("mha_d128", 3, 2, 2, 128, [300, 1, 64], [257, 300, 1], 256),
    ("gqa2_d64", 4, 4, 2, 64, [129, 64, 2, 31], [65, 200, 128, 1], 100),
    ("gqa3_d128", 2, 6, 2, 128, [100, 7], [120, 170], 85),
    ("gqa16_d64", 2, 16, 1, 64, [50, 3], [40, 90], 16),
    ("one_token_steps", 2, 8, 2, 128, [65, 1], [5, 3], 1),
]


@pytest.mark.parametrize("name,B,Hq,Hkv,D,P,R,C", CASES, ids=[c[0] for c in CASES])
def test_shapes_and_ragged_tails(gpu, name, B, Hq, Hkv, D, P, R, C):
    cfg = small_cfg(B, Hq, Hkv, D, C, seed=4321 + B * 7 + Hq)
    ep = build_episode(cfg, threads=2, lengths=(np.array(P, np.int32), np.array(R, np.int32)))
    run_and_check(gpu, ep, oracle_uniform_chunks(ep.prompt_len, ep.resp_len, C), None, name)


@pytest.mark.parametrize("split,order", [(1, 0), (2, 0), (3, 1), (7, 2), (64, 0)])
def test_split_kv_and_order_do_not_change_results(gpu, split, order):
    binding, episode, torch = gpu
    cfg = small_cfg(4, 8, 2, 128, 96, seed=99)
    ep = build_episode(cfg, threads=2, lengths=(np.array([700, 64, 1, 330], np.int32), np.array([200, 96, 333, 10], np.int32)))
    ref = oracle_outputs(ep)
    binding.oppo_set_option(binding.OPT_SPLIT_KV, split)
    binding.oppo_set_option(binding.OPT_ORDER, order)
    try:
        run_and_check(gpu, ep, oracle_uniform_chunks(ep.prompt_len, ep.resp_len, 96), ref, f"split={split} order={order}")
    finally:
        binding.oppo_set_option(binding.OPT_SPLIT_KV, 0)
        binding.oppo_set_option(binding.OPT_ORDER, 0)


@pytest.mark.parametrize("G,D,split", [(1, 128, 0), (3, 128, 0), (4, 128, 3), (5, 64, 0), (8, 128, 0), (16, 64, 3)])
def test_short_tiles_leave_waves_without_rows(gpu, G, D, split):
    """Steps whose chunks fill 1, 2, ... of the 8 waves' 32-row blocks of a packed tile
    (a tile of n tokens has n * G rows), next to full tiles, on contexts of several
    key tiles: every count of waves with rows occurs, with the key range whole and cut."""
    binding, episode, torch = gpu
    tm = 256 // G
    per_wave = max(1, 32 // G)
    q_lens = sorted({1, per_wave, per_wave + 1, 3 * per_wave, 5 * per_wave - 1, tm - 1, tm, tm + 1})
    B = len(q_lens)
    P = np.array([130 + 37 * i for i in range(B)], np.int32)
    R = np.array([3 * q for q in q_lens], np.int32)
    cfg = small_cfg(B, 2 * G, 2, D, 64, seed=700 + G)
    ep = build_episode(cfg, threads=2, lengths=(P, R))
    # prompts first, then three steps in which sequence i gets q_lens[(i + step) % B] rows
    chunks = [[int(p) for p in P]]
    left = R.astype(np.int64).copy()
    step = 0
    while left.any():
        take = [int(min(left[i], q_lens[(i + step) % B])) for i in range(B)]
        left -= np.array(take)
        chunks.append(take)
        step += 1
    binding.oppo_set_option(binding.OPT_SPLIT_KV, split)
    try:
        run_and_check(gpu, ep, chunks, None, f"short tiles G={G} D={D} split={split}")
    finally:
        binding.oppo_set_option(binding.OPT_SPLIT_KV, 0)


def test_empty_batch_and_all_finished(gpu):
    binding, episode, torch = gpu
    cfg = small_cfg(3, 8, 2, 128, 32)
    ep = build_episode(cfg, threads=1, lengths=(np.array([10, 20, 30], np.int32), np.array([5, 5, 5], np.int32)))
    chunks = [[10, 20, 30], [0, 0, 0], [5, 0, 5], [0, 5, 0], [0, 0, 0]]
    run_and_check(gpu, ep, chunks, None, "zero-length passes")


@pytest.mark.parametrize("split", [0, 1, 3])
def test_late_dominant_keys_rerun_in_exact_mode(gpu, split):
    """Keys far into a sequence that outscore its first keys by a wide margin: the
    kernel's first run of such a piece (weights against the maximum of the first 32
    keys) sees row sums beyond its limit - or plain overflow - and the piece is run
    again in the exact mode.  Results must still match the oracle."""
    binding, episode, torch = gpu
    cfg = small_cfg(3, 8, 2, 128, 128, seed=4321)
    P, R = np.array([70, 300, 33], np.int32), np.array([200, 140, 128], np.int32)
    ep = build_episode(cfg, threads=1, lengths=(P, R))
    one, four, sixteen, minus2 = 0x3F80, 0x4080, 0x4180, 0xC000
    for i, spots in enumerate([[(45, four), (150, sixteen)], [(299, four), (310, minus2), (400, sixteen)], [(100, sixteen)]]):
        lo = int(ep.tok_begin[i])
        ep.q[lo:int(ep.tok_begin[i + 1])] = one          # every query is the all-ones vector
        for pos, val in spots:
            ep.k[lo + pos] = val                         # score = 128 * val * scale: +45, +181 (overflow), -23
    binding.oppo_set_option(binding.OPT_SPLIT_KV, split)
    try:
        for C in (128, 64):
            run_and_check(gpu, ep, oracle_uniform_chunks(P, R, C), None, f"dominant keys C={C} split={split}")
    finally:
        binding.oppo_set_option(binding.OPT_SPLIT_KV, 0)


def test_causality_within_last_chunk(gpu):
    """Perturb the last tokens of the final chunk: earlier rows of the same
    chunk, computed in the same launch with the same work list, do not change
    by a single bit."""
    binding, episode, torch = gpu
    cfg = small_cfg(2, 8, 2, 128, 128, seed=77)
    P, R = np.array([100, 257], np.int32), np.array([128, 128], np.int32)
    ep = build_episode(cfg, threads=1, lengths=(P, R))
    chunks = oracle_uniform_chunks(P, R, 128)
    _, base, _ = run_and_check(gpu, ep, chunks)
    ep2 = build_episode(cfg, threads=1, lengths=(P, R))
    cut = 77  # perturb response tokens >= cut of every sequence
    for i in range(2):
        lo = int(ep2.tok_begin[i]) + int(P[i]) + cut
        hi = int(ep2.tok_begin[i + 1])
        for arr in (ep2.q, ep2.k, ep2.v):
            arr[lo:hi] ^= np.uint16(0x8055)  # sign and low mantissa bits: magnitudes stay N(0,1)-like
    _, pert, _ = run_and_check(gpu, ep2, chunks)
    for i in range(2):
        lo = int(ep.tok_begin[i])
        mid = lo + int(P[i]) + cut
        assert np.array_equal(base[lo:mid], pert[lo:mid])
        assert not np.array_equal(base[mid:int(ep.tok_begin[i + 1])], pert[mid:int(ep.tok_begin[i + 1])])


def test_capacity_error_writes_nothing(gpu):
    binding, episode, torch = gpu
    desc = binding.make_desc(8, 2, 128, 0.1)
    ck = torch.full((20, 2, 128), -1, dtype=torch.int16, device="cuda:0")
    cv = ck.clone()
    cache = binding.KVCache(ck, cv, np.array([0, 8, 20]), np.array([6, 0]))
    new = torch.ones((6, 2, 128), dtype=torch.int16, device="cuda:0")
    with pytest.raises(binding.OppoError) as e:
        binding.oppo_kv_append(desc, cache, [0, 3, 6], new, new)   # seq 0: 6 + 3 > 8
    assert e.value.code == binding.OPPO_ERR_CAPACITY
    torch.cuda.synchronize()
    assert cache.kv_len.tolist() == [6, 0]
    assert bool((ck == -1).all()) and bool((cv == -1).all())
    binding.oppo_kv_append(desc, cache, [0, 2, 6], new, new)      # fits exactly
    torch.cuda.synchronize()
    assert cache.kv_len.tolist() == [8, 4]
    assert bool((ck[6:8] == 1).all()) and bool((ck[8:12] == 1).all()) and bool((ck[12:] == -1).all())
    assert bool((ck[:6] == -1).all())


def test_snapshot_restore_resumes_identically(gpu):
    """The cache is the resumable state: copy slabs + lengths after a pass,
    run on, restore, run again -> identical bits."""
    binding, episode, torch = gpu
    cfg = small_cfg(3, 8, 2, 128, 40, seed=5)
    ep = build_episode(cfg, threads=1, lengths=(np.array([90, 10, 64], np.int32), np.array([100, 130, 7], np.int32)))
    chunks = oracle_uniform_chunks(ep.prompt_len, ep.resp_len, 40)
    se = episode.StreamedEpisode(ep, chunks)
    se.run_step(0)
    se.run_step(1)
    torch.cuda.synchronize()
    snap_k, snap_v, snap_len = se.cache_k.clone(), se.cache_v.clone(), se.cache.kv_len.copy()
    for t in range(2, len(chunks)):
        se.run_step(t)
    torch.cuda.synchronize()
    first = [s.out.clone() for s in se.steps]
    final_k = se.cache_k.clone()
    se.cache_k.copy_(snap_k)
    se.cache_v.copy_(snap_v)
    se.cache.kv_len[:] = snap_len
    for s in se.steps[2:]:
        s.out.zero_()
    for t in range(2, len(chunks)):
        se.run_step(t)
    torch.cuda.synchronize()
    for a, s in zip(first, se.steps):
        assert torch.equal(a, s.out)
    assert torch.equal(final_k, se.cache_k)


@pytest.mark.parametrize("gain,split", [(4.0, 0), (4.0, 3), (8.0, 0)])
def test_peaked_softmax_moves_the_reference_often(gpu, gain, split):
    """Queries and keys scaled up so that logits spread over +-40 nats and more: the weights
    of a column span hundreds of bits, and the running reference of the softmax has to be
    moved again and again in the middle of pieces, of the tile that straddles the cache
    boundary in the fused call, and of split pieces that are merged with very different
    references.  (Inputs are N(0,1) bf16 times a power of two: still exact bf16.)"""
    binding, episode, torch = gpu
    cfg = small_cfg(3, 8, 2, 128, 80, seed=2718)
    ep = build_episode(cfg, threads=2, lengths=(np.array([300, 70, 1], np.int32), np.array([260, 500, 90], np.int32)))
    scale_bits = int(np.log2(gain)) << 7                        # bf16 exponent field starts at bit 7
    for t in (ep.q, ep.k):
        nz = (t & 0x7F80) != 0                                  # zeros and subnormals stay as they are
        t[nz] = (t[nz] + scale_bits).astype(np.uint16)
    binding.oppo_set_option(binding.OPT_SPLIT_KV, split)
    try:
        se, out, (mx, mean) = run_and_check(gpu, ep, oracle_uniform_chunks(ep.prompt_len, ep.resp_len, cfg.chunk), None,
                                            f"peaked gain={gain} split={split}")
    finally:
        binding.oppo_set_option(binding.OPT_SPLIT_KV, 0)
    print(f"peaked softmax gain {gain}: max abs err {mx:.3e}, mean {mean:.3e}")
