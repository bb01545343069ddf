#!/usr/bin/env python3
"""Benchmark of the streamed chunked-prefill path on one MI355X.

One "step" is one streamed episode of the workload: every pass t = 0..T-1 of
the streaming loop (Alg. 1, generation loop; Sec. 3.1), each pass being one
oppo_chunk_step (KV append fused into the chunked-prefill attention; with
--two-call: oppo_kv_append followed by oppo_chunk_prefill_attn) over the ragged
set of unfinished sequences.  Prompts are prefilled once before the timed
region (reported separately).  Inputs are synthetic and resident in HBM.

Prints ONE JSON line: `value` = algorithmic attention FLOPs of the episode per
second of wall time over the timed episodes (TFLOP/s); `roofline` = the
attention kernel alone (FLOPs, or bytes on a workload the memory roof binds,
per second of kernel time measured with HIP events on the launch stream,
against the chip's published peak; `traffic` = HBM bytes per launch measured
with rocprofv3 counters); `cpu_baseline` = the float64 oracle timed on a bounded
sample of the same workload.  Other modes (--deferral, --chunk-sweep, --overlap,
--inter-step, --contention) print one JSON line of their own.
"""
from __future__ import annotations

import argparse
import dataclasses
import gc
import json
import os
import sys
import time

import numpy as np
from typing import List

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E
# HBM bytes per attention launch (reads + writes) from rocprofv3 FETCH_SIZE / WRITE_SIZE,
# scaled by what the same counters read for the append kernel (a plain copy of known
# size); see profiles/attn_fwd_kernel_config2.md and profiles/attn_fwd_kernel_config3_traffic.md.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = {2: 259.5e6, 3: 523.6e6}


@dataclasses.dataclass(frozen=True)
class TimingModel:
    """Synthetic timing of what surrounds the measured attention passes: the generating
    side (actor) and the dense part of the scorer's layers.  Stated figures, not
    measurements - they stand in for the 8B-class models of the paper's runs (Sec. 4.1)
    on one accelerator each, and only give the measured attention time something to be
    hidden behind (Sec. 3.1):
      * a decode step of the actor is bound by memory traffic: all weights plus the
        K/V of every live token are read once per generated token;
      * every chunk boundary costs the actor a fixed hand-off (synchronise, ship the
        chunk's tokens, launch the scorer's pass) - the cost that grows as chunks
        shrink (Sec. 3.1, "Dynamic Control on Intra-step Overlap");
      * the scorer's projections and MLPs cost a fixed number of FLOPs per token.
    """
    layers: int = 32
    weight_bytes: float = 2 * 8.03e9                  # bf16 parameters
    kv_bytes_per_token: float = 2 * 32 * 8 * 128 * 2  # K and V, 32 layers x 8 kv-heads x 128, bf16
    decode_bytes_per_s: float = 5.0e12
    decode_step_overhead_s: float = 30e-6
    handoff_s: float = 2e-3
    dense_flops_per_token: float = 2 * 8.03e9
    dense_flops_per_s: float = 1.2e15

    def decode_step_s(self, live_tokens: float) -> float:
        return self.decode_step_overhead_s + (self.weight_bytes + live_tokens * self.kv_bytes_per_token) / self.decode_bytes_per_s

    def dense_s(self, tokens: float) -> float:
        return tokens * self.dense_flops_per_token / self.dense_flops_per_s


def generation_times(prompt_len, resp_len, C: int, model: TimingModel) -> List[float]:
    """Seconds the modelled actor needs for each chunk of C decode steps (the last chunk
    may be shorter), with every unfinished sequence of the batch decoding in lockstep."""
    P = np.asarray(prompt_len, dtype=np.int64)
    R = np.asarray(resp_len, dtype=np.int64)
    out: List[float] = []
    longest = int(R.max()) if len(R) else 0
    for c0 in range(0, longest, C):
        t = model.handoff_s
        for j in range(c0, min(c0 + C, longest)):
            live = R > j
            t += model.decode_step_s(float((P[live] + j).sum()))
        out.append(t)
    return out


def pass_generation_time(kv_before, q_len, model: TimingModel) -> float:
    """Seconds the modelled actor needs to produce one pass's rows: sequence i decodes
    q_len[i] tokens on top of kv_before[i], all in lockstep, each step reading the
    weights and the K/V of the sequences still decoding; plus one hand-off."""
    kvb = np.asarray(kv_before, dtype=np.int64)
    ql = np.asarray(q_len, dtype=np.int64)
    t = model.handoff_s
    for j in range(int(ql.max()) if len(ql) else 0):
        live = ql > j
        t += model.decode_step_s(float((kvb[live] + j).sum()))
    return t


def cpu_baseline(cfg, ep, budget_s: float = 12.0):
    """Times the float64 oracle, as it stands, on a bounded sample: whole
    sequences of the workload (one-shot causal attention over prompt+response,
    all heads; only the response rows' share of the FLOPs is credited), taken
    in order of closeness to the median length until the time budget is spent."""
    from oracle import bf16_bits_to_f64, causal_attention
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    n = ep.prompt_len.astype(np.int64) + ep.resp_len
    order = np.argsort(np.abs(n - np.median(n)), kind="stable")
    flops = 0.0
    used = []
    t0 = time.perf_counter()
    for i in order:
        lo = int(ep.tok_begin[i])
        P, R = int(ep.prompt_len[i]), int(ep.resp_len[i])
        q = bf16_bits_to_f64(ep.q[lo + P:lo + P + R])
        k = bf16_bits_to_f64(ep.k[lo:lo + P + R])
        v = bf16_bits_to_f64(ep.v[lo:lo + P + R])
        causal_attention(q, k, v, P + np.arange(R), cfg.softmax_scale)
        flops += 4.0 * cfg.head_dim * cfg.num_q_heads * (R * P + R * (R + 1) / 2.0)
        used.append(int(i))
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    return {
        "value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
        "sample": f"{len(used)} of {cfg.batch} sequences nearest the median length, response rows x all heads, "
                  f"float64 numpy, {dt:.1f} s",
    }


def chunk_sweep(args, cfg, torch, ob) -> int:
    """The intra-step trade-off in the scorer's own terms (Sec. 3.1; Sec. 4.3, impact of streaming degrees):
    small chunks cost GPU time (more passes, more fixed cost per pass), large chunks leave a long last
    pass that starts only when generation has ended and so cannot be hidden behind it."""
    from paper_2509_25762_amd.episode import StreamedEpisode, uniform_chunks
    from paper_2509_25762_amd.workload import build_episode, episode_work
    ep = build_episode(cfg, threads=min(16, len(os.sched_getaffinity(0))))
    candidates = [64, 128, 256, 512, 1024]
    rows = []
    for C in candidates:
        chunks = uniform_chunks(ep.prompt_len, ep.resp_len, C)
        T = len(chunks) - 1
        copies = [StreamedEpisode(ep, chunks) for _ in range(2)]
        work = episode_work(dataclasses.replace(cfg, chunk=C), [(s.kv_before, s.q_len) for s in copies[0].steps[1:]])
        flops = sum(w["flops"] for w in work)
        for se in copies:
            se.reset(0)
            se.run_step(0)

        def episode(se):
            se.reset(1)
            for t in range(1, T + 1):
                se.run_step(t)

        steps, warmup = max(8, args.steps // 4), max(8, args.warmup // 2)
        for w in range(warmup):
            episode(copies[w % 2])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s_ in range(steps):
            episode(copies[s_ % 2])
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        # the last pass on its own (library events around its launches)
        ob.oppo_profile_enable(True)
        last = 0.0
        for s_ in range(8):
            se = copies[s_ % 2]
            se.reset(1)
            for t in range(1, T):
                se.run_step(t)
            ob.oppo_profile_read()
            se.run_step(T)
            kms, _ = ob.oppo_profile_read()
            last += (kms["attn"] + kms["merge"]) / 8
        ob.oppo_profile_enable(False)
        rows.append({"chunk": C, "passes": T, "episode_ms": ms, "tflops": flops / (ms * 1e-3) / 1e12, "last_pass_ms": last})
        del copies
        torch.cuda.empty_cache()
    # the tuner, fed with (scorer time that competes with generation for the GPU) + (tail that cannot overlap)
    tuner = ob.oppo_tuner_create(candidates, 50)
    picked = None
    for step in range(len(candidates) + 1):
        c = ob.oppo_tuner_chunk(tuner, step)
        r = rows[candidates.index(c)]
        ob.oppo_tuner_report(tuner, step, (r["episode_ms"] + r["last_pass_ms"]) * 1e-3)
        picked = c
    ob.oppo_tuner_destroy(tuner)
    print(json.dumps({"metric": "streamed episode vs chunk size", "config": {"workload": f"config {cfg.index} ({cfg.name}) lengths, "
                      f"B={cfg.batch}, chunk sizes {candidates}"}, "sweep": rows,
                      "tuner_objective": "episode_ms + last_pass_ms", "tuner_pick": picked, "n_gpus": 1, "data": "synthetic"}))
    return 0


def overlap_study(args, cfg, torch, ob) -> int:
    """Intra-step overlap in the paper's own quantity (Sec. 3.1): how much of the scorer's time is
    hidden behind generation, and the step time that results, per chunk size.  The scorer's
    attention passes are measured here (library events around each pass's kernels, times the
    model's layer count); the generating side and the dense part of the scorer's layers come from
    the stated synthetic model (TimingModel above).  The two sides are taken to run on separate
    accelerators.  The prompts are chunk 0 of the timeline, complete at time 0 (they are known before
    generation starts).  Baseline: generation, then one prefill of everything."""
    from paper_2509_25762_amd.episode import StreamedEpisode, uniform_chunks
    from paper_2509_25762_amd.workload import build_episode
    model = TimingModel()
    ep = build_episode(cfg, threads=min(16, len(os.sched_getaffinity(0))))
    candidates = [16, 32, 64, 128, 256, 512, 1024, 2048, 4096]
    reps = 5
    ob.oppo_profile_enable(True)
    resp_tokens = float(np.sum(ep.resp_len))
    all_tokens = float(np.sum(ep.prompt_len) + np.sum(ep.resp_len))
    # baseline scoring: one prefill of prompt + response
    se = StreamedEpisode(ep, uniform_chunks(ep.prompt_len, ep.resp_len, 1 << 20))
    once_ms = 0.0
    for r in range(reps + 1):
        ob.oppo_profile_read()
        se.full_prefill()
        kms, _ = ob.oppo_profile_read()
        if r:
            once_ms += (kms["attn"] + kms["merge"]) / reps
    del se
    torch.cuda.empty_cache()
    score_once_s = model.layers * once_ms * 1e-3 + model.dense_s(all_tokens)
    rows = []
    for C in candidates:
        chunks = uniform_chunks(ep.prompt_len, ep.resp_len, C)
        T = len(chunks) - 1
        se = StreamedEpisode(ep, chunks)
        pass_ms = np.zeros(T + 1)
        for r in range(reps + 1):
            se.reset(0)
            for t in range(T + 1):
                ob.oppo_profile_read()
                se.run_step(t)
                kms, _ = ob.oppo_profile_read()
                if r:
                    pass_ms[t] += (kms["attn"] + kms["merge"] + kms["append"]) / reps
        gen_s = [0.0] + generation_times(ep.prompt_len, ep.resp_len, C, model)
        assert len(gen_s) == T + 1
        tokens = np.array([float(np.sum(st.q_len)) for st in se.steps])
        score_s = model.layers * pass_ms * 1e-3 + np.array([model.dense_s(x) for x in tokens])
        _, _, summ = ob.oppo_overlap_timeline(gen_s, score_s)
        sequential = float(np.sum(gen_s)) - (T - 1) * model.handoff_s + score_once_s   # one hand-off, at the end
        rows.append({"chunk": C, "passes": T, "generation_s": float(np.sum(gen_s)), "scoring_s": float(np.sum(score_s)),
                     "attention_s": float(model.layers * pass_ms.sum() * 1e-3), "exposed_s": summ["exposed"],
                     "hidden_frac": 1.0 - summ["exposed"] / float(np.sum(score_s)), "step_s": summ["step_end"],
                     "sequential_s": sequential, "speedup": sequential / summ["step_end"]})
        del se
        torch.cuda.empty_cache()
    ob.oppo_profile_enable(False)
    tuner = ob.oppo_tuner_create(candidates, 50)
    picked = None
    for step in range(len(candidates) + 1):
        c = ob.oppo_tuner_chunk(tuner, step)
        ob.oppo_tuner_report(tuner, step, rows[candidates.index(c)]["step_s"])
        picked = c
    ob.oppo_tuner_destroy(tuner)
    print(json.dumps({"metric": "modelled step time with intra-step overlap vs chunk size",
                      "config": {"workload": f"config {cfg.index} ({cfg.name}) lengths, B={cfg.batch}, chunk sizes {candidates}"},
                      "model": dataclasses.asdict(model), "score_once_attention_ms_per_layer": once_ms,
                      "sweep": rows, "tuner_pick": picked, "n_gpus": 1, "data": "synthetic",
                      "note": "attention passes measured, everything else from the stated model; response tokens "
                              f"{int(resp_tokens)}, all tokens {int(all_tokens)}"}))
    return 0


def inter_step_study(args, cfg, torch, ob) -> int:
    """Inter-step overlap in the paper's own quantity (Sec. 3.2, Alg. 1): time to turn a dataset into
    PPO batches of B sequences when the buffer holds B + Delta, so that an iteration ends with the
    B-th finisher instead of the slowest sequence and the unfinished ones carry their cached prefix
    over.  Every pass of the library's scheduler / slot pool / fused attention call is measured
    (library events, x the model's layer count); generation and the scorer's dense work come from the
    stated synthetic model (TimingModel above); each iteration is one intra-step timeline
    (oppo_overlap_timeline), iterations follow one another (the PPO update in between is the same
    for every Delta and left out).  Baseline: Delta = 0 without streaming (generate, then score once)."""
    from paper_2509_25762_amd.episode import BufferedRun
    from paper_2509_25762_amd.workload import build_episode
    model = TimingModel()
    B = cfg.batch
    n_seq = 4 * B
    ep = build_episode(dataclasses.replace(cfg, batch=n_seq), threads=min(16, len(os.sched_getaffinity(0))))
    reps = 3
    rows = []
    ob.oppo_profile_enable(True)
    for delta in (0, 4, 8, 16, 32):
        run = BufferedRun(ep, B, delta, cfg.chunk)
        passes = run.passes()
        pass_ms = np.zeros(len(passes))
        for r in range(reps + 1):
            run.reset()
            k = 0
            for e in run.events:
                if e[0] == "acquire":
                    ob.oppo_pool_acquire(run.pool, e[1], e[2])
                elif e[0] == "release":
                    ob.oppo_pool_release(run.pool, e[1])
                elif e[0] == "pass":
                    ps = e[1]
                    ob.oppo_profile_read()
                    ob.oppo_chunk_step(run.desc, run.cache, ps.cu_q, ps.q, ps.k, ps.v, ps.out, run.workspace)
                    kms, _ = ob.oppo_profile_read()
                    if r:
                        pass_ms[k] += (kms["attn"] + kms["merge"] + kms["append"]) / reps
                    k += 1
        n_iter = len(run.removed)
        tot = {"generation_s": 0.0, "scoring_s": 0.0, "exposed_s": 0.0, "step_s": 0.0, "sequential_s": 0.0}
        for it in range(n_iter):
            idx = [k for k, ps in enumerate(passes) if ps.iteration == it]
            gen = [0.0 if passes[k].kind == ob.PASS_PROMPT else pass_generation_time(passes[k].kv_before, passes[k].q_len, model)
                   for k in idx]
            score = [model.layers * pass_ms[k] * 1e-3 + model.dense_s(float(np.sum(passes[k].q_len))) for k in idx]
            _, _, summ = ob.oppo_overlap_timeline(gen, score)
            tot["generation_s"] += float(np.sum(gen))
            tot["scoring_s"] += float(np.sum(score))
            tot["exposed_s"] += summ["exposed"]
            tot["step_s"] += summ["step_end"]
            n_chunk = sum(1 for k in idx if passes[k].kind != ob.PASS_PROMPT)
            tot["sequential_s"] += float(np.sum(gen)) - max(0, n_chunk - 1) * model.handoff_s + float(np.sum(score))
        rows.append({"delta": delta, "slots": B + delta, "iterations": n_iter, "passes": len(passes),
                     "attention_s": float(model.layers * pass_ms.sum() * 1e-3), **tot,
                     "sequences_per_s": n_seq / tot["step_s"]})
        del run
        torch.cuda.empty_cache()
    ob.oppo_profile_enable(False)
    base = rows[0]["sequential_s"]
    for r in rows:
        r["speedup_vs_sequential"] = base / r["step_s"]
        r["speedup_vs_streaming_only"] = rows[0]["step_s"] / r["step_s"]
    print(json.dumps({"metric": "modelled time for a dataset with inter-step overlap vs Delta",
                      "config": {"workload": f"config {cfg.index} ({cfg.name}) lengths, {n_seq} sequences, PPO batch B={B}, "
                                             f"C={cfg.chunk}, buffer of B + Delta slots"},
                      "model": dataclasses.asdict(model), "baseline": "Delta = 0, generate then score (sequential_s of the first row)",
                      "rows": rows, "n_gpus": 1, "data": "synthetic",
                      "note": "attention passes measured, everything else from the stated model"}))
    return 0


def rope_bench(args, cfg, torch, ob) -> int:
    """The rotary embedding of a pass's rows (oppo_rope), HBM-bound: every q and k row of the
    workload's first response pass is read and written once.  Timed with events on the launch
    stream; each launch turns the same rows once more (the values stay finite: a rotation)."""
    from paper_2509_25762_amd.workload import draw_lengths
    P, R = draw_lengths(cfg)
    q_len = np.minimum(cfg.chunk, R).astype(np.int32)
    cu = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int32)
    rows = int(cu[-1])
    dev = torch.device("cuda:0")
    # several copies taken in turn: together larger than the chip's 256 MB last-level cache, so that
    # every launch finds its rows in HBM
    ncopy = max(1, args.copies)
    qs = [torch.randn((rows, cfg.num_q_heads, cfg.head_dim), device=dev, dtype=torch.bfloat16).view(torch.int16) for _ in range(ncopy)]
    ks = [torch.randn((rows, cfg.num_kv_heads, cfg.head_dim), device=dev, dtype=torch.bfloat16).view(torch.int16) for _ in range(ncopy)]
    desc = ob.make_desc(cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.softmax_scale)
    steps, warmup = max(20, args.steps), max(10, args.warmup)
    for i in range(warmup):
        ob.oppo_rope(desc, P, cu, qs[i % ncopy], ks[i % ncopy])
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(steps):
        ob.oppo_rope(desc, P, cu, qs[i % ncopy], ks[i % ncopy])
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    nbytes = 2.0 * rows * (cfg.num_q_heads + cfg.num_kv_heads) * cfg.head_dim * 2
    print(json.dumps({"metric": "rotary embedding of a pass's q and k rows, in place", "value": nbytes / (ms * 1e-3) / 1e9,
                      "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms, "higher_is_better": True,
                      "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"config {cfg.index} ({cfg.name}), first response pass: {rows} rows x "
                                             f"({cfg.num_q_heads} + {cfg.num_kv_heads}) heads x {cfg.head_dim}, {ncopy} copies in turn"},
                      "roofline": {"bound": "hbm", "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                   "frac": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, "traffic": None, "kernel": "rope_kernel",
                                   "algorithmic_bytes_per_launch": nbytes}}))
    return 0


def qkv_epilogue_bench(args, cfg, torch, ob) -> int:
    """oppo_qkv_rope_append on the workload's first response pass: one pass over the projection's
    output rows [q | k | v], rotated queries out, rotated keys and values into the cache.  HBM-bound:
    every byte read once and written once.  Several copies in turn, as for --rope."""
    from paper_2509_25762_amd.workload import draw_lengths
    P, R = draw_lengths(cfg)
    q_len = np.minimum(cfg.chunk, R).astype(np.int32)
    cu = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int32)
    rows = int(cu[-1])
    dev = torch.device("cuda:0")
    heads = cfg.num_q_heads + 2 * cfg.num_kv_heads
    ncopy = max(1, args.copies)
    slot_begin = np.concatenate([[0], np.cumsum(P.astype(np.int64) + q_len)])
    qkvs = [torch.randn((rows, heads, cfg.head_dim), device=dev, dtype=torch.bfloat16).view(torch.int16) for _ in range(ncopy)]
    q_outs = [torch.empty((rows, cfg.num_q_heads, cfg.head_dim), device=dev, dtype=torch.int16) for _ in range(ncopy)]
    caches = []
    for _ in range(ncopy):
        ck = torch.zeros((int(slot_begin[-1]), cfg.num_kv_heads, cfg.head_dim), device=dev, dtype=torch.int16)
        caches.append(ob.KVCache(ck, torch.zeros_like(ck), slot_begin, P))
    desc = ob.make_desc(cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.softmax_scale)
    steps, warmup = max(20, args.steps), max(10, args.warmup)

    def call(i):
        c = caches[i % ncopy]
        c.kv_len[:] = P                        # the same pass again
        ob.oppo_qkv_rope_append(desc, c, cu, qkvs[i % ncopy], q_outs[i % ncopy])

    for i in range(warmup):
        call(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(steps):
        call(i)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    nbytes = 2.0 * rows * heads * cfg.head_dim * 2
    print(json.dumps({"metric": "QKV-projection epilogue: rotary embedding + cache write in one pass", "value": nbytes / (ms * 1e-3) / 1e9,
                      "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms, "higher_is_better": True,
                      "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"config {cfg.index} ({cfg.name}), first response pass: {rows} rows x "
                                             f"({cfg.num_q_heads} + 2 x {cfg.num_kv_heads}) heads x {cfg.head_dim}, {ncopy} copies in turn"},
                      "roofline": {"bound": "hbm", "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                   "frac": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, "traffic": None,
                                   "kernel": "qkv_rope_append_kernel", "algorithmic_bytes_per_launch": nbytes}}))
    return 0


def layer_path_bench(args, cfg, torch, ob) -> int:
    """The attention side of one scorer layer over the streamed episode, two ways:
      A  oppo_rope in place on the chunk's q and k rows, then oppo_chunk_step (append fused into attention);
      B  oppo_qkv_rope_append over the projection's output rows [q | k | v] (rotated keys and values straight
         into the cache), then oppo_chunk_prefill_attn.
    Both give the same outputs up to the tolerance (same rotated values, same attention); timed like the
    main benchmark (prompts prefilled before the timed region, cache copies taken in turn)."""
    from paper_2509_25762_amd.episode import StreamedEpisode, uniform_chunks
    from paper_2509_25762_amd.workload import build_episode, episode_work
    ep = build_episode(cfg, threads=min(16, len(os.sched_getaffinity(0))))
    chunks = uniform_chunks(ep.prompt_len, ep.resp_len, cfg.chunk)
    T = len(chunks) - 1
    copies = [StreamedEpisode(ep, chunks) for _ in range(max(1, args.copies))]
    work = episode_work(cfg, [(s.kv_before, s.q_len) for s in copies[0].steps[1:]])
    flops = sum(w["flops"] for w in work)
    for se in copies:
        se.reset(0)
        se.run_step(0)
        # inputs of path B: the projection's output rows, and a place for the rotated queries; path A
        # rotates q and k in place, so it works on copies of its own (rotated again every episode:
        # the values stay finite, and the timing does not depend on them)
        se.qkv = [torch.cat([st.q, st.k, st.v], dim=1).contiguous() for st in se.steps]
        se.q_rot = [torch.empty_like(st.q) for st in se.steps]
        se.qa = [st.q.clone() for st in se.steps]
        se.ka = [st.k.clone() for st in se.steps]

    def path_a(se):
        se.reset(1)
        for t in range(1, T + 1):
            st = se.steps[t]
            ob.oppo_rope(se.desc, st.kv_before, st.cu_q, se.qa[t], se.ka[t])
            ob.oppo_chunk_step(se.desc, se.cache, st.cu_q, se.qa[t], se.ka[t], st.v, st.out, se.workspace)

    def path_b(se):
        se.reset(1)
        for t in range(1, T + 1):
            st = se.steps[t]
            ob.oppo_qkv_rope_append(se.desc, se.cache, st.cu_q, se.qkv[t], se.q_rot[t])
            ob.oppo_chunk_prefill_attn(se.desc, se.cache, st.cu_q, se.q_rot[t], st.out, se.workspace)

    res = {}
    for name, fn in (("rope_in_place_then_chunk_step", path_a), ("qkv_epilogue_then_attention", path_b)):
        for w in range(args.warmup):
            fn(copies[w % len(copies)])
        torch.cuda.synchronize()
        gc.collect()
        gc.disable()
        t0 = time.perf_counter()
        for s_ in range(args.steps):
            fn(copies[s_ % len(copies)])
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        gc.enable()
        res[name] = {"ms_per_episode": ms, "attention_tflops": flops / (ms * 1e-3) / 1e12}
    print(json.dumps({"metric": "attention side of one scorer layer over the streamed episode", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "data": "synthetic", "dtype": "bf16",
                      "config": {"workload": f"config {cfg.index} ({cfg.name}): B={cfg.batch}, C={cfg.chunk}, {T} passes per episode"},
                      "paths": res}))
    return 0


def thin_pass_bench(args, cfg, torch, ob) -> int:
    """Passes with very few new rows per sequence on long contexts (the last chunk of a response,
    a one-token pass for the final score): the query tile has 1 or 16 tokens x G heads, so most of
    the workgroup's waves have no rows and only move key tiles; the pass is bound by reading K and V.
    Uniform batches with the workload's head shape; K/V of all sequences exceed the last-level cache."""
    dev = torch.device("cuda:0")
    Hq, Hkv, D = cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim
    desc = ob.make_desc(Hq, Hkv, D, cfg.softmax_scale)
    rows = []
    for B, kv_before, q_len in ((64, 4095, 1), (256, 2047, 1), (64, 16383, 1), (64, 4080, 16), (64, 16368, 16)):
        cap = kv_before + q_len
        slot_begin = np.arange(B + 1, dtype=np.int64) * cap
        ck = torch.randn((B * cap, Hkv, D), device=dev, dtype=torch.bfloat16).view(torch.int16)
        cv = torch.randn((B * cap, Hkv, D), device=dev, dtype=torch.bfloat16).view(torch.int16)
        q = torch.randn((B * q_len, Hq, D), device=dev, dtype=torch.bfloat16).view(torch.int16)
        out = torch.empty_like(q)
        cache = ob.KVCache(ck, cv, slot_begin, np.full(B, cap, dtype=np.int32))
        cu = (np.arange(B + 1) * q_len).astype(np.int32)
        ws = torch.empty(ob.oppo_workspace_bytes(desc, B, B * q_len), dtype=torch.uint8, device=dev)
        steps, warmup = max(50, args.steps), max(20, args.warmup)
        for _ in range(warmup):
            ob.oppo_chunk_prefill_attn(desc, cache, cu, q, out, ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        gc.collect()
        gc.disable()
        e0.record()
        for _ in range(steps):
            ob.oppo_chunk_prefill_attn(desc, cache, cu, q, out, ws)
        e1.record()
        torch.cuda.synchronize()
        gc.enable()
        ms = e0.elapsed_time(e1) / steps
        kv_bytes = 2.0 * B * cap * Hkv * D * 2          # every key and value row of every sequence, once
        rows.append({"batch": B, "kv_before": kv_before, "q_len": q_len, "ms": ms, "kv_GBps": kv_bytes / (ms * 1e-3) / 1e9,
                     "frac_of_hbm_peak": kv_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBPS})
        del ck, cv, q, out, ws
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "thin passes: K/V read rate of oppo_chunk_prefill_attn with 1 or 16 new rows per sequence",
                      "unit": "GB/s", "n_gpus": 1, "data": "synthetic", "dtype": "bf16",
                      "config": {"workload": f"uniform batches, Hq/Hkv/D={Hq}/{Hkv}/{D}"}, "rows": rows}))
    return 0


def steady_bench(args, cfg, torch, ob) -> int:
    """The attention call on uniform batches with long contexts (no raggedness, whole tiles, every
    queue equally long): the kernel's steady state, to set beside the stand-alone instruction-mix
    loop of ceiling_bench.  One chunk of the workload's size C on top of 8K - C and 1K - C cached tokens."""
    from paper_2509_25762_amd.workload import step_work
    dev = torch.device("cuda:0")
    Hq, Hkv, D, C = cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.chunk
    desc = ob.make_desc(Hq, Hkv, D, cfg.softmax_scale)
    rows = []
    for B, total in ((64, 8192), (64, 1024)):
        kv_before, q_len = max(total, 2 * C) - C, C
        cap = kv_before + q_len
        slot_begin = np.arange(B + 1, dtype=np.int64) * cap
        ck = torch.randn((B * cap, Hkv, D), device=dev, dtype=torch.bfloat16).view(torch.int16)
        cv = torch.randn((B * cap, Hkv, D), device=dev, dtype=torch.bfloat16).view(torch.int16)
        q = torch.randn((B * q_len, Hq, D), device=dev, dtype=torch.bfloat16).view(torch.int16)
        out = torch.empty_like(q)
        cache = ob.KVCache(ck, cv, slot_begin, np.full(B, cap, dtype=np.int32))
        cu = (np.arange(B + 1) * q_len).astype(np.int32)
        ws = torch.empty(ob.oppo_workspace_bytes(desc, B, B * q_len), dtype=torch.uint8, device=dev)
        steps, warmup = max(10, args.steps // 4), max(20, args.warmup)
        for _ in range(warmup):
            ob.oppo_chunk_prefill_attn(desc, cache, cu, q, out, ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        gc.collect()
        gc.disable()
        e0.record()
        for _ in range(steps):
            ob.oppo_chunk_prefill_attn(desc, cache, cu, q, out, ws)
        e1.record()
        torch.cuda.synchronize()
        gc.enable()
        ms = e0.elapsed_time(e1) / steps
        w = step_work(cfg, np.full(B, kv_before), np.full(B, q_len))
        rows.append({"batch": B, "kv_before": kv_before, "q_len": q_len, "ms": ms, "tflops": w["flops"] / (ms * 1e-3) / 1e12,
                     "frac_of_mfma_peak": w["flops"] / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                     "kv_GBps": w["kv_read_bytes"] / (ms * 1e-3) / 1e9})
        del ck, cv, q, out, ws
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "steady state of oppo_chunk_prefill_attn on uniform batches", "unit": "TFLOP/s", "n_gpus": 1,
                      "data": "synthetic", "dtype": "bf16",
                      "config": {"workload": f"uniform batches, Hq/Hkv/D={Hq}/{Hkv}/{D}, one chunk of {C} rows per sequence"},
                      "rows": rows}))
    return 0


def contention_study(args, cfg, torch, ob) -> int:
    """The scorer's chunked prefill next to a generation-like load on the same GPU (Sec. 3.1: with
    colocated models small chunks risk contention).  The attention kernel runs one persistent workgroup
    per compute unit it is given, so the split of the chip is a launch parameter: with fewer CUs for the
    scorer, the other stream's kernels find free CUs instead of waiting for whole launches to end."""
    from paper_2509_25762_amd.episode import StreamedEpisode, uniform_chunks
    from paper_2509_25762_amd.workload import build_episode, episode_work
    dev = torch.device("cuda:0")
    ep = build_episode(cfg, threads=min(16, len(os.sched_getaffinity(0))))
    chunks = uniform_chunks(ep.prompt_len, ep.resp_len, cfg.chunk)
    T = len(chunks) - 1
    copies = [StreamedEpisode(ep, chunks) for _ in range(2)]
    work = episode_work(cfg, [(s.kv_before, s.q_len) for s in copies[0].steps[1:]])
    flops = sum(w["flops"] for w in work)
    for se in copies:
        se.reset(0)
        se.run_step(0)
    # decode-like load: a sweep over 16 weight matrices of 8192 x 8192 bf16 (2 GiB in all), one
    # matrix-vector product each - bound by reading the weights, like a decoding step at small batch
    W = [torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16) for _ in range(16)]
    x = torch.randn(8192, device=dev, dtype=torch.bfloat16)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()

    def attn(n):
        for i in range(n):
            se = copies[i % 2]
            se.reset(1)
            for t in range(1, T + 1):
                se.run_step(t, stream=sa)

    def decode(n):
        with torch.cuda.stream(sb):
            for _ in range(n):
                for w in W:
                    torch.mv(w, x)

    def timed(fa, fb, na, nb):
        torch.cuda.synchronize()
        ea0, ea1, eb0, eb1 = (torch.cuda.Event(enable_timing=True) for _ in range(4))
        ea0.record(sa), eb0.record(sb)
        # enqueue in small slices so that both streams always have work queued
        ia = ib = 0
        while ia < na or ib < nb:
            if ia < na and fa:
                fa(min(4, na - ia))
            ia += 4
            if ib < nb and fb:
                fb(min(4, nb - ib))
            ib += 4
        ea1.record(sa), eb1.record(sb)
        torch.cuda.synchronize()
        return ea0.elapsed_time(ea1), eb0.elapsed_time(eb1)

    def masked_streams(n_attn):
        """Two streams whose kernels may only run on disjoint sets of compute units: mask bits
        [0, n_attn) for the scorer, the rest for the other load (hipExtStreamCreateWithCUMask; default
        priority).  Returns None if the runtime refuses."""
        import ctypes
        hip = ctypes.CDLL("libamdhip64.so")
        out = []
        for lo, hi in ((0, n_attn), (n_attn, 256)):
            words = (ctypes.c_uint32 * 8)(*[sum(1 << b for b in range(32) if lo <= 32 * w + b < hi) for w in range(8)])
            h = ctypes.c_void_p()
            if hip.hipExtStreamCreateWithCUMask(ctypes.byref(h), 8, words) != 0 or not h.value:
                return None
            out.append(torch.cuda.ExternalStream(h.value))
        return out

    rows = []
    n_ep, n_dec = 120, 60
    plain = (sa, sb)
    for cus, masked in ((256, False), (192, False), (128, False), (192, True), (128, True)):
        if masked:
            pair = masked_streams(cus)
            if pair is None:
                rows.append({"attention_cus": cus, "cu_masks": "refused by the runtime"})
                continue
            sa, sb = pair
        else:
            sa, sb = plain
        ob.oppo_set_option(ob.OPT_NUM_CUS, cus)
        timed(attn, decode, 40, 20)                      # warm-up
        a_alone, _ = timed(attn, None, n_ep, 0)
        _, d_alone = timed(None, decode, 0, n_dec)
        a_both, d_both = timed(attn, decode, n_ep, n_dec)
        rows.append({"attention_cus": cus, "cu_masks": bool(masked),
                     "episode_ms_alone": a_alone / n_ep, "episode_ms_colocated": a_both / n_ep,
                     "tflops_alone": flops / (a_alone / n_ep * 1e-3) / 1e12,
                     "tflops_colocated": flops / (a_both / n_ep * 1e-3) / 1e12,
                     "decode_sweep_ms_alone": d_alone / n_dec, "decode_sweep_ms_colocated": d_both / n_dec,
                     "decode_GBps_alone": 16 * 8192 * 8192 * 2 / (d_alone / n_dec * 1e-3) / 1e9,
                     "decode_GBps_colocated": 16 * 8192 * 8192 * 2 / (d_both / n_dec * 1e-3) / 1e9})
    ob.oppo_set_option(ob.OPT_NUM_CUS, 256)
    print(json.dumps({"metric": "colocation of chunked prefill with a memory-bound load", "n_gpus": 1, "data": "synthetic",
                      "config": {"workload": f"config {cfg.index} ({cfg.name}) episode on one stream; 16 x (8192 x 8192 bf16 "
                                             "matrix-vector product) sweeps on another; default stream priorities"},
                      "rows": rows}))
    return 0


def deferral_bench(args, cfg, torch, ob) -> int:
    """Alg. 1 with B + Delta slots over a dataset of 2 x batch sequences (see --deferral)."""
    from paper_2509_25762_amd.episode import BufferedRun
    from paper_2509_25762_amd.workload import build_episode, episode_work
    delta = args.deferral
    if delta >= cfg.batch:
        print("bench.py: --deferral needs DELTA < batch", file=sys.stderr)
        return 2
    data_cfg = dataclasses.replace(cfg, batch=2 * cfg.batch)
    ep = build_episode(data_cfg, threads=min(16, len(os.sched_getaffinity(0))))
    B = cfg.batch - delta
    runs = [BufferedRun(ep, B, delta, cfg.chunk) for _ in range(2)]
    passes = runs[0].passes()
    work = episode_work(cfg, [(p.kv_before, p.q_len) for p in passes])
    flops = sum(w["flops"] for w in work)
    tot_bytes = sum(w["kv_read_bytes"] + w["qo_bytes"] + w["append_bytes"] for w in work)
    steps, warmup = max(1, args.steps // 4), max(1, args.warmup // 4)   # a run is ~4 episodes' worth of work
    for w in range(warmup):
        runs[w % 2].reset()
        runs[w % 2].run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        runs[s % 2].reset()
        runs[s % 2].run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    ob.oppo_profile_enable(True)
    ob.oppo_profile_read()
    prof_steps = min(steps, 12)
    for s in range(prof_steps):
        runs[s % 2].reset()
        runs[s % 2].run()
    kms, n = ob.oppo_profile_read()
    ob.oppo_profile_enable(False)
    achieved = flops / (kms["attn"] / prof_steps * 1e-3) / 1e12
    n_iter = len(runs[0].removed)
    line = {
        "metric": "chunked-prefill attn TFLOP/s + KV GB/s, % of MI355X roofline, 1 GPU",
        "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"config {cfg.index} ({cfg.name}) with inter-step overlap: {2 * cfg.batch} sequences through "
                               f"{cfg.batch} cache slots, B={B}, Delta={delta}, C={cfg.chunk}, {n_iter} iterations, "
                               f"{len(passes)} passes (prompt passes included), {int(sum(w['rows'] for w in work))} rows",
                   "step": "the whole run: slot acquisitions, one oppo_chunk_step per pass, releases",
                   "slot_reuses": int(runs[0].pool_counts[3])},
        "total_GBps": tot_bytes / (ms * 1e-3) / 1e9,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None, "kernel": "attn_fwd_kernel",
                     "launches_per_step": n["attn"] / prof_steps,
                     "avg_launch_ms": kms["attn"] / max(1, n["attn"])},
        "merge_kernel_ms_per_step": kms["merge"] / prof_steps,
        "cpu_baseline": None,
    }
    print(json.dumps(line))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200, help="timed episodes (about 0.2 s: long enough for the clocks to settle under load)")
    ap.add_argument("--warmup", type=int, default=50, help="untimed episodes; the core clock needs tens of milliseconds of load to settle")
    ap.add_argument("--config", type=int, default=2, help="workload index 1..5 (default: the Llama-3-8B-shape layer)")
    ap.add_argument("--copies", type=int, default=4, help="independent cache copies rotated between episodes")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-workspace", action="store_true", help="disable split-KV")
    ap.add_argument("--split", type=int, default=0, help="split-KV policy (0 auto, 1 off, n forced)")
    ap.add_argument("--details", type=str, default="", help="write per-pass details to this JSON file")
    ap.add_argument("--deferral", type=int, default=-1, metavar="DELTA",
                    help="inter-step overlap instead of one episode: a dataset of twice the workload's sequences "
                         "streamed through batch cache slots, B = batch - DELTA of which finish per iteration "
                         "(Alg. 1); every pass, the prompts' included, is one oppo_chunk_step over all slots")
    ap.add_argument("--chunk-sweep", action="store_true",
                    help="time the workload's streamed episode for chunk sizes 64..1024 (total scorer time and the "
                         "last pass, which cannot overlap generation) and let the chunk-size tuner pick")
    ap.add_argument("--overlap", action="store_true",
                    help="intra-step overlap as a timeline: measured attention passes of the scorer (x 32 layers) "
                         "against a stated synthetic model of the generating side, per chunk size 16..2048: "
                         "hidden fraction of the scoring time, step time, speed-up over generate-then-score")
    ap.add_argument("--inter-step", action="store_true",
                    help="inter-step overlap as a timeline: 4 x batch sequences turned into PPO batches through a buffer "
                         "of batch + Delta slots (Alg. 1) for Delta = 0..32; measured scorer passes against the stated "
                         "synthetic model of the generating side; time per dataset and speed-up over Delta = 0")
    ap.add_argument("--rope", action="store_true",
                    help="time oppo_rope (rotary embedding of a pass's q and k rows) on the workload's first response pass")
    ap.add_argument("--qkv-epilogue", action="store_true",
                    help="time oppo_qkv_rope_append (rotary embedding + cache write as one pass over the QKV projection's "
                         "output) on the workload's first response pass")
    ap.add_argument("--layer-path", action="store_true",
                    help="the streamed episode with the rotary embedding included, two ways: oppo_rope + oppo_chunk_step, "
                         "and oppo_qkv_rope_append + oppo_chunk_prefill_attn")
    ap.add_argument("--thin-pass", action="store_true",
                    help="attention passes with 1 or 16 new rows per sequence on contexts of 2K-16K tokens: K/V read rate")
    ap.add_argument("--steady", action="store_true",
                    help="the attention call on uniform batches (64 sequences, one chunk on top of 8K and 1K contexts): "
                         "the kernel's steady state")
    ap.add_argument("--contention", action="store_true",
                    help="colocation study: the streamed episode on one stream and a memory-bound decode-like load "
                         "(bf16 matrix-vector products) on another, alone and together, with the attention launch "
                         "restricted to 256 / 192 / 128 compute units (OPPO_OPT_NUM_CUS), without and with CU masks on the two streams")
    ap.add_argument("--two-call", action="store_true",
                    help="oppo_kv_append + oppo_chunk_prefill_attn per pass instead of the fused oppo_chunk_step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2509_25762_amd import binding as ob
    from paper_2509_25762_amd.episode import StreamedEpisode, uniform_chunks
    from paper_2509_25762_amd.workload import CONFIGS, build_episode, episode_work

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    ob.load()
    if args.split:
        ob.oppo_set_option(ob.OPT_SPLIT_KV, args.split)
    cfg = CONFIGS[args.config]
    if args.deferral >= 0:
        return deferral_bench(args, cfg, torch, ob)
    if args.chunk_sweep:
        return chunk_sweep(args, cfg, torch, ob)
    if args.overlap:
        return overlap_study(args, cfg, torch, ob)
    if args.inter_step:
        return inter_step_study(args, cfg, torch, ob)
    if args.rope:
        return rope_bench(args, cfg, torch, ob)
    if args.qkv_epilogue:
        return qkv_epilogue_bench(args, cfg, torch, ob)
    if args.layer_path:
        return layer_path_bench(args, cfg, torch, ob)
    if args.thin_pass:
        return thin_pass_bench(args, cfg, torch, ob)
    if args.steady:
        return steady_bench(args, cfg, torch, ob)
    if args.contention:
        return contention_study(args, cfg, torch, ob)
    ep = build_episode(cfg, threads=min(16, len(os.sched_getaffinity(0))))
    chunks = uniform_chunks(ep.prompt_len, ep.resp_len, cfg.chunk)
    T = len(chunks) - 1
    copies = [StreamedEpisode(ep, chunks, use_workspace=not args.no_workspace) for _ in range(max(1, args.copies))]
    # shared inputs are identical across copies; only the cache slabs and outputs differ
    work = episode_work(cfg, [(s.kv_before, s.q_len) for s in copies[0].steps[1:]])
    flops = sum(w["flops"] for w in work)
    kv_bytes = sum(w["kv_read_bytes"] for w in work)
    tot_bytes = sum(w["kv_read_bytes"] + w["qo_bytes"] + w["append_bytes"] for w in work)

    # prompt prefill, once per copy, timed on its own
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for se in copies:
        se.reset(0)
        se.run_step(0)
    torch.cuda.synchronize()
    prompt_ms = (time.perf_counter() - t0) * 1e3 / len(copies)

    fused = not args.two_call

    def episode(se):
        se.reset(1)
        for t in range(1, T + 1):
            se.run_step(t, fused=fused)

    for w in range(args.warmup):
        episode(copies[w % len(copies)])
    torch.cuda.synchronize()
    # (a full pass of Python's cyclic garbage collector over the imported modules takes tens of
    # milliseconds of host time, during which nothing is enqueued: none inside the timed region)
    gc.collect()
    gc.disable()
    t0 = time.perf_counter()
    for s in range(args.steps):
        episode(copies[s % len(copies)])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    gc.enable()
    ms_per_step = dt * 1e3 / args.steps

    # kernel-level timing: the library brackets each of its kernel launches with HIP
    # events on the launch stream (the stream the kernels run on).  The episodes are
    # enqueued back to back like the timed ones and the events are read once at the
    # end, so the kernels are timed at the clock rate the sustained load settles at.
    prof_steps = min(args.steps, 50)
    ob.oppo_profile_enable(True)
    ob.oppo_profile_read()
    for s in range(prof_steps):
        episode(copies[s % len(copies)])
    ms, n = ob.oppo_profile_read()
    attn_total_ms = ms["attn"] / prof_steps
    launches_per_step = n["attn"] / prof_steps
    achieved = flops / (attn_total_ms * 1e-3) / 1e12
    attn_ms = merge_ms = app_ms = None
    if args.details:
        # per pass: the events are read after every pass, which idles the GPU in between
        attn_ms = np.zeros((prof_steps, T))
        merge_ms = np.zeros((prof_steps, T))
        app_ms = np.zeros((prof_steps, T))
        for s in range(prof_steps):
            se = copies[s % len(copies)]
            se.reset(1)
            for t in range(1, T + 1):
                se.run_step(t, fused=fused)
                pm, _ = ob.oppo_profile_read()
                attn_ms[s, t - 1], merge_ms[s, t - 1], app_ms[s, t - 1] = pm["attn"], pm["merge"], pm["append"]
    ob.oppo_profile_enable(False)

    tflops = flops / (ms_per_step * 1e-3) / 1e12
    # which roof binds the attention kernel on this workload (classical roofline over the episode's launches)
    bound = "mfma" if flops / (PEAK_BF16_TFLOPS * 1e12) >= tot_bytes / (PEAK_HBM_GBPS * 1e9) else "hbm"
    achieved_gbps = tot_bytes / (attn_total_ms * 1e-3) / 1e9
    t_roof_ms = sum(max(w["flops"] / (PEAK_BF16_TFLOPS * 1e12),
                        (w["kv_read_bytes"] + w["qo_bytes"] + w["append_bytes"]) / (PEAK_HBM_GBPS * 1e9)) for w in work) * 1e3
    line = {
        "metric": "chunked-prefill attn TFLOP/s + KV GB/s, % of MI355X roofline, 1 GPU",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"config {cfg.index} ({cfg.name}): B={cfg.batch}, Hq/Hkv/D={cfg.num_q_heads}/"
                               f"{cfg.num_kv_heads}/{cfg.head_dim}, C={cfg.chunk}, {T} passes per episode, "
                               f"{int(sum(w['rows'] for w in work))} response rows",
                   "step": ("one streamed episode (one oppo_chunk_step per pass: KV append + chunked-prefill attention)"
                            if fused else "one streamed episode (oppo_kv_append + oppo_chunk_prefill_attn per pass)"),
                   "cache_copies_rotated": len(copies)},
        "kv_read_GBps": kv_bytes / (ms_per_step * 1e-3) / 1e9,
        "total_GBps": tot_bytes / (ms_per_step * 1e-3) / 1e9,
        "frac_of_roofline_episode": t_roof_ms / ms_per_step,
        "frac_mfma_peak": tflops / PEAK_BF16_TFLOPS,
        "frac_hbm_peak": tot_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBPS,
        "prompt_prefill_ms": prompt_ms,
        "roofline": {"bound": bound, "achieved": achieved if bound == "mfma" else achieved_gbps,
                     "peak": PEAK_BF16_TFLOPS if bound == "mfma" else PEAK_HBM_GBPS,
                     "unit": "TFLOP/s" if bound == "mfma" else "GB/s",
                     "frac": achieved / PEAK_BF16_TFLOPS if bound == "mfma" else achieved_gbps / PEAK_HBM_GBPS,
                     "traffic": MEASURED_TRAFFIC_BYTES_PER_LAUNCH.get(cfg.index),
                     "algorithmic_bytes_per_launch": sum(w["kv_read_bytes"] + w["qo_bytes"] +
                                                         (w["append_bytes"] if fused else 0) for w in work) / T,
                     "kernel": "attn_fwd_kernel",
                     "launches_per_step": launches_per_step, "avg_launch_ms": attn_total_ms / launches_per_step},
        "append_kernel_ms_per_step": ms["append"] / prof_steps,
        "merge_kernel_ms_per_step": ms["merge"] / prof_steps,
    }
    if args.details:
        attn_pass_ms = attn_ms.mean(axis=0)
        det = {"attn_pass_ms": attn_pass_ms.tolist(), "append_pass_ms": app_ms.mean(axis=0).tolist(),
               "merge_pass_ms": merge_ms.mean(axis=0).tolist(),
               "work": work, "ms_per_step": ms_per_step}
        with open(args.details, "w") as f:
            json.dump(det, f, indent=1)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg, ep)
    else:
        line["cpu_baseline"] = None
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
