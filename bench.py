#!/usr/bin/env python3
"""Benchmark of the streamed chunked-prefill path on one MI355X.

One "step" is one streamed episode of the workload: every pass t = 0..T-1 of
the streaming loop (Alg. 1, generation loop; Sec. 3.1), each pass being one
oppo_chunk_step (KV append fused into the chunked-prefill attention; with
--two-call: oppo_kv_append followed by oppo_chunk_prefill_attn) over the ragged
set of unfinished sequences.  Prompts are prefilled once before the timed
region (reported separately).  Inputs are synthetic and resident in HBM.

Prints ONE JSON line.  Headline = the Llama-3-8B-shape workload (config 2):
`value` = algorithmic attention FLOPs of the episode per second of wall time over
the timed episodes (TFLOP/s); `roofline` = the attention kernel alone (FLOPs, or
bytes on a workload the memory roof binds, per second of kernel time measured
with HIP events on the launch stream, against the chip's published peak;
`traffic` = HBM bytes per launch measured with rocprofv3 counters, read from
profiles/hbm_traffic.json); `step0` = the full-batch first pass on its own;
`pass_cold` = the same episodes interleaved pass by pass over the cache copies,
so that no pass finds the previous pass's keys in the last-level cache;
`host_us_per_pass` = what a pass costs on the host; `per_config` = the other
synthetic workloads measured the same way (and a parity bit for the tiny one);
`cpu_baseline` = the float64 oracle timed on a bounded sample of the headline
workload, single-threaded and over a process pool.  Before any timed region the
GPU is kept busy until at least SETTLE_MS of load have run, whatever --warmup
says: after idling, the core clock needs tens of milliseconds of load to settle.
Other modes (--deferral, --chunk-sweep, --overlap, --inter-step, --contention,
--traffic-from ...) print one JSON line of their own.
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
PEAK_FP8_TFLOPS = 5000.0    # MI355X dense fp8 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E
SETTLE_MS = 200.0            # load the GPU has seen before a timed region starts, at least
# HBM bytes per attention launch (reads + writes) from rocprofv3 FETCH_SIZE / WRITE_SIZE, scaled by
# what the same counters read for a plain copy of known size: written by `bench.py --traffic-from`
# into this file together with a fingerprint of the kernel and planner sources it was measured on.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
TRAFFIC_SOURCES = ["paper_2509_25762_amd/csrc/kernels.hip", "paper_2509_25762_amd/csrc/api.cpp",
                   "paper_2509_25762_amd/csrc/oppo_internal.h"]


def source_fingerprint() -> str:
    """Hash of the sources that decide how many bytes a launch moves (kernel, planner)."""
    import hashlib
    h = hashlib.sha256()
    for rel in TRAFFIC_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(config_index: int):
    """(bytes per launch or None, note): the tracked measurement if it was taken on these sources."""
    try:
        with open(TRAFFIC_FILE) as f:
            data = json.load(f)
    except (OSError, ValueError):
        return None, "no tracked measurement (profiles/hbm_traffic.json missing)"
    entry = data.get("configs", {}).get(str(config_index))
    if entry is None:
        return None, "not measured for this workload"
    if data.get("source_fingerprint") != source_fingerprint():
        return None, f"stale: measured at commit {data.get('commit', '?')} on other kernel/planner sources"
    return float(entry["traffic_bytes_per_launch"]), f"measured at commit {data.get('commit', '?')}"


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


def _oracle_unit(job):
    """One (sequence, q-head) unit of the oracle: the response rows of that head over the head's keys."""
    from oracle import bf16_bits_to_f64, causal_attention
    qb, kb, vb, P, R, scale = job
    causal_attention(bf16_bits_to_f64(qb), bf16_bits_to_f64(kb), bf16_bits_to_f64(vb), P + np.arange(R), scale)
    return 4.0 * qb.shape[-1] * (R * P + R * (R + 1) / 2.0)


def cpu_baseline(cfg, ep, budget_s: float = 8.0):
    """Times the float64 oracle, as it stands, on a bounded sample of the workload, two ways:
    single-threaded (BLAS limited to one thread) over whole sequences nearest the median length
    (one-shot causal attention over prompt + response, all heads; only the response rows' share of
    the FLOPs is credited), and with a process pool over (sequence, q-head) units on all cores the
    process may use.  Must run before this process touches the GPU (the pool forks)."""
    import multiprocessing as mp
    from oracle import bf16_bits_to_f64, causal_attention
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threadpool_limits = None
        blas_threads = None
    cores = len(os.sched_getaffinity(0))
    n = ep.prompt_len.astype(np.int64) + ep.resp_len
    order = np.argsort(np.abs(n - np.median(n)), kind="stable")

    def seq_arrays(i):
        lo = int(ep.tok_begin[i])
        P, R = int(ep.prompt_len[i]), int(ep.resp_len[i])
        return ep.q[lo + P:lo + P + R], ep.k[lo:lo + P + R], ep.v[lo:lo + P + R], P, R

    def single():
        flops, used, t0 = 0.0, 0, time.perf_counter()
        for i in order:
            qb, kb, vb, P, R = seq_arrays(i)
            causal_attention(bf16_bits_to_f64(qb), bf16_bits_to_f64(kb), bf16_bits_to_f64(vb), P + np.arange(R), cfg.softmax_scale)
            flops += 4.0 * cfg.head_dim * cfg.num_q_heads * (R * P + R * (R + 1) / 2.0)
            used += 1
            if time.perf_counter() - t0 > budget_s:
                break
        return flops, used, time.perf_counter() - t0

    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            f1, n1, dt1 = single()
    else:
        f1, n1, dt1 = single()
    # process pool: units of one (sequence, q-head), handed out until the budget is spent
    G = cfg.num_q_heads // cfg.num_kv_heads
    workers = max(1, cores)

    def units():
        for i in order:
            qb, kb, vb, P, R = seq_arrays(i)
            for h in range(cfg.num_q_heads):
                g = h // G
                yield (np.ascontiguousarray(qb[:, h:h + 1]), np.ascontiguousarray(kb[:, g:g + 1]),
                       np.ascontiguousarray(vb[:, g:g + 1]), P, R, cfg.softmax_scale)

    fp, np_units, t0 = 0.0, 0, time.perf_counter()
    if threadpool_limits is not None:
        limiter = threadpool_limits(limits=1)     # inherited by the forked workers: one BLAS thread each
    with mp.get_context("fork").Pool(workers) as pool:
        for got in pool.imap_unordered(_oracle_unit, units(), chunksize=1):
            fp += got
            np_units += 1
            if time.perf_counter() - t0 > budget_s:
                pool.terminate()
                break
    dtp = time.perf_counter() - t0
    if threadpool_limits is not None:
        limiter.restore_original_limits()
    return {
        "value": fp / dtp / 1e12, "unit": "TFLOP/s", "cores": int(workers), "kind": "oracle",
        "sample": f"process pool of {workers} workers (one BLAS thread each) over {np_units} (sequence, q-head) units of the "
                  f"sequences nearest the median length, response rows, float64 numpy, {dtp:.1f} s",
        "single_thread": {"value": f1 / dt1 / 1e12, "unit": "TFLOP/s", "cores": 1,
                          "sample": f"{n1} whole sequences nearest the median length, all heads, {dt1:.1f} s"},
        "affinity_cores": int(cores), "blas_threads": blas_threads,
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


def qkv_proj_measure(args, cfg, torch, ob, only_fused=False):
    """The layer's fused QKV projection on the workload's first response pass, two ways:
      fused    oppo_qkv_proj_rope_append: hand-written MFMA GEMM whose epilogue rotates queries and keys and writes
               keys and values into the cache (the projection's output never exists in memory);
      library  torch.matmul (the vendor library's GEMM) writing [q | k | v] rows, then oppo_qkv_rope_append over them.
    hidden = Hq * D (a square attention block, 4096 for the Llama-3-8B shape); synthetic weights ~ N(0, 1/hidden)."""
    from paper_2509_25762_amd.workload import draw_lengths
    P, R = draw_lengths(cfg)
    q_len = np.minimum(cfg.chunk, R).astype(np.int32)
    cu = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int32)
    rows = int(cu[-1])
    dev = torch.device("cuda:0")
    Hq, Hkv, D = cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim
    hidden = Hq * D
    n_out = (Hq + 2 * Hkv) * D
    ncopy = max(1, args.copies)
    slot_begin = np.concatenate([[0], np.cumsum(P.astype(np.int64) + q_len)])
    xs = [torch.randn((rows, hidden), device=dev, dtype=torch.bfloat16) for _ in range(ncopy)]
    w = (torch.randn((n_out, hidden), device=dev, dtype=torch.float32) / np.sqrt(hidden)).to(torch.bfloat16)
    q_outs = [torch.empty((rows, Hq, D), device=dev, dtype=torch.int16) for _ in range(ncopy)]
    ys = [torch.empty((rows, n_out), device=dev, dtype=torch.bfloat16) for _ in range(ncopy)]
    caches = []
    for _ in range(ncopy):
        ck = torch.zeros((int(slot_begin[-1]), Hkv, D), device=dev, dtype=torch.int16)
        caches.append(ob.KVCache(ck, torch.zeros_like(ck), slot_begin, P))
    desc = ob.make_desc(Hq, Hkv, D, cfg.softmax_scale)
    ws = torch.empty(ob.oppo_qkv_proj_workspace_bytes(desc, rows), dtype=torch.uint8, device=dev)
    steps, warmup = max(20, args.steps // 4), max(10, args.warmup // 2)

    def fused(i):
        c = caches[i % ncopy]
        c.kv_len[:] = P
        ob.oppo_qkv_proj_rope_append(desc, c, cu, xs[i % ncopy].view(torch.int16), hidden, w.view(torch.int16), q_outs[i % ncopy], ws)

    def library(i):
        c = caches[i % ncopy]
        c.kv_len[:] = P
        torch.matmul(xs[i % ncopy], w.t(), out=ys[i % ncopy])
        ob.oppo_qkv_rope_append(desc, c, cu, ys[i % ncopy].view(torch.int16).view(rows, Hq + 2 * Hkv, D), q_outs[i % ncopy])

    def gemm_only(i):
        torch.matmul(xs[i % ncopy], w.t(), out=ys[i % ncopy])

    flops = 2.0 * rows * hidden * n_out
    res = {}
    paths = (("fused_projection_rope_append", fused), ("library_gemm_then_rope_append", library), ("library_gemm_alone", gemm_only))
    for name, fn in paths[:1] if only_fused else paths:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        done, total = 0, 0.0
        while total < SETTLE_MS:                          # settle the clocks under this very load
            e0.record()
            for _ in range(warmup):
                fn(done)
                done += 1
            e1.record()
            e1.synchronize()
            total += e0.elapsed_time(e1)
        e0.record()
        for i in range(steps):
            fn(done + i)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        res[name] = {"ms": ms, "tflops": flops / (ms * 1e-3) / 1e12, "frac_of_mfma_peak": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
    workload = (f"config {cfg.index} ({cfg.name}), first response pass: {rows} rows x hidden {hidden} -> "
                f"({Hq} + 2 x {Hkv}) heads x {D}, {ncopy} copies in turn")
    return res, workload, steps, warmup


def qkv_proj_rows_sweep(args, cfg, torch, ob) -> int:
    """Fused projection against library GEMM + oppo_qkv_rope_append for passes of 256 .. 16384 rows (uniform
    sequences of 256 new rows on empty caches, the configuration's head shape, hidden = Hq * D): the pass sizes
    a streamed episode goes through as its batch thins out.  The launch picks its tile height per pass."""
    dev = torch.device("cuda:0")
    Hq, Hkv, D = cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim
    hidden, n_out, C = Hq * D, (Hq + 2 * Hkv) * D, 256
    desc = ob.make_desc(Hq, Hkv, D, cfg.softmax_scale)
    w = (torch.randn((n_out, hidden), device=dev, dtype=torch.float32) / np.sqrt(hidden)).to(torch.bfloat16)
    out = []
    for B in (1, 2, 4, 8, 16, 32, 64):
        rows = B * C
        P = np.zeros(B, dtype=np.int32)
        cu = (np.arange(B + 1) * C).astype(np.int32)
        ck = torch.zeros((rows, Hkv, D), device=dev, dtype=torch.int16)
        cache = ob.KVCache(ck, torch.zeros_like(ck), np.arange(B + 1, dtype=np.int64) * C, P)
        q_out = torch.empty((rows, Hq, D), device=dev, dtype=torch.int16)
        y = torch.empty((rows, n_out), device=dev, dtype=torch.bfloat16)
        xs = [torch.randn((rows, hidden), device=dev, dtype=torch.bfloat16) for _ in range(3)]
        ws = torch.empty(ob.oppo_qkv_proj_workspace_bytes(desc, rows), dtype=torch.uint8, device=dev)

        def fused(i):
            cache.kv_len[:] = P
            ob.oppo_qkv_proj_rope_append(desc, cache, cu, xs[i % 3].view(torch.int16), hidden, w.view(torch.int16), q_out, ws)

        def library(i):
            cache.kv_len[:] = P
            torch.matmul(xs[i % 3], w.t(), out=y)
            ob.oppo_qkv_rope_append(desc, cache, cu, y.view(torch.int16).view(rows, Hq + 2 * Hkv, D), q_out)

        row = {"rows": rows}
        for name, fn in (("fused_ms", fused), ("library_gemm_then_rope_append_ms", library)):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            done, total = 0, 0.0
            while total < SETTLE_MS / 2:
                e0.record()
                for _ in range(20):
                    fn(done)
                    done += 1
                e1.record()
                e1.synchronize()
                total += e0.elapsed_time(e1)
            e0.record()
            for i in range(50):
                fn(done + i)
            e1.record()
            torch.cuda.synchronize()
            row[name] = e0.elapsed_time(e1) / 50
        row["fused_tflops"] = 2.0 * rows * hidden * n_out / (row["fused_ms"] * 1e-3) / 1e12
        out.append(row)
    print(json.dumps({"metric": "fused QKV projection over pass sizes", "unit": "ms", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"passes of 256 new rows per sequence, hidden {hidden} -> ({Hq} + 2 x {Hkv}) heads x {D}"},
                      "passes": out}))
    return 0


def qkv_proj_bench(args, cfg, torch, ob) -> int:
    if args.rows_sweep:
        return qkv_proj_rows_sweep(args, cfg, torch, ob)
    res, workload, steps, warmup = qkv_proj_measure(args, cfg, torch, ob)
    f = res["fused_projection_rope_append"]
    print(json.dumps({"metric": "fused QKV projection with rotary / cache epilogue", "value": f["tflops"], "unit": "TFLOP/s", "n_gpus": 1,
                      "steps": steps, "warmup": warmup, "ms_per_step": f["ms"], "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": workload},
                      "roofline": {"bound": "mfma", "achieved": f["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                                   "frac": f["frac_of_mfma_peak"], "traffic": None, "kernel": "qkv_proj_kernel"},
                      "paths": res}))
    return 0


def layer_path_bench(args, cfg, torch, ob) -> int:
    """The attention side of one scorer layer over the streamed episode, two ways (and, with the layer's QKV
    projection included, two more: oppo_qkv_proj_rope_append + attention against the vendor library's GEMM +
    oppo_qkv_rope_append + attention):
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

    # with the projection included: hidden rows of every pass (synthetic, hidden = Hq * D) and the layer's weights
    hidden = cfg.num_q_heads * cfg.head_dim
    n_out = (cfg.num_q_heads + 2 * cfg.num_kv_heads) * cfg.head_dim
    dev = torch.device("cuda:0")
    w = (torch.randn((n_out, hidden), device=dev, dtype=torch.float32) / np.sqrt(hidden)).to(torch.bfloat16)
    for se in copies:
        se.x = [torch.randn((int(st.cu_q[-1]), hidden), device=dev, dtype=torch.bfloat16) for st in se.steps]
        se.y = [torch.empty((int(st.cu_q[-1]), n_out), device=dev, dtype=torch.bfloat16) for st in se.steps]
    max_rows = max(int(st.cu_q[-1]) for st in copies[0].steps)
    proj_ws = torch.empty(ob.oppo_qkv_proj_workspace_bytes(copies[0].desc, max_rows), dtype=torch.uint8, device=dev)
    heads = cfg.num_q_heads + 2 * cfg.num_kv_heads

    def path_c(se):
        se.reset(1)
        for t in range(1, T + 1):
            st = se.steps[t]
            ob.oppo_qkv_proj_rope_append(se.desc, se.cache, st.cu_q, se.x[t].view(torch.int16), hidden, w.view(torch.int16), se.q_rot[t], proj_ws)
            ob.oppo_chunk_prefill_attn(se.desc, se.cache, st.cu_q, se.q_rot[t], st.out, se.workspace)

    def path_d(se):
        se.reset(1)
        for t in range(1, T + 1):
            st = se.steps[t]
            torch.matmul(se.x[t], w.t(), out=se.y[t])
            ob.oppo_qkv_rope_append(se.desc, se.cache, st.cu_q, se.y[t].view(torch.int16).view(-1, heads, cfg.head_dim), se.q_rot[t])
            ob.oppo_chunk_prefill_attn(se.desc, se.cache, st.cu_q, se.q_rot[t], st.out, se.workspace)

    res = {}
    for name, fn in (("rope_in_place_then_chunk_step", path_a), ("qkv_epilogue_then_attention", path_b),
                     ("fused_projection_then_attention", path_c), ("library_gemm_then_qkv_epilogue_then_attention", path_d)):
        done, total = 0, 0.0
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        while total < SETTLE_MS:
            e0.record()
            for _ in range(max(1, args.warmup // 4)):
                fn(copies[done % len(copies)])
                done += 1
            e1.record()
            e1.synchronize()
            total += e0.elapsed_time(e1)
        steps = args.steps if name.startswith(("rope", "qkv")) else max(10, args.steps // 5)
        torch.cuda.synchronize()
        gc.collect()
        gc.disable()
        t0 = time.perf_counter()
        for s_ in range(steps):
            fn(copies[s_ % len(copies)])
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
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
    ap.add_argument("--qkv-proj", action="store_true",
                    help="time the fused QKV projection with its rotary / cache epilogue (oppo_qkv_proj_rope_append) on the "
                         "workload's first response pass, next to the vendor library's GEMM followed by oppo_qkv_rope_append")
    ap.add_argument("--rows-sweep", action="store_true",
                    help="with --qkv-proj: passes of 256 .. 16384 rows instead of the workload's first pass")
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
    ap.add_argument("--single", action="store_true", help="only the workload named by --config, no per_config block")
    ap.add_argument("--traffic-from", type=str, default="", metavar="DIR",
                    help="no GPU work: read rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE csv files from DIR and write profiles/hbm_traffic.json")
    ap.add_argument("--fp8-cache", action="store_true",
                    help="study: the workload of --config through the 16-bit cache (append + attention "
                         "calls) and through the cache of 8-bit codes, same protocol, one JSON line")
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

    cfg = CONFIGS[args.config]
    special = (args.deferral >= 0 or args.chunk_sweep or args.overlap or args.inter_step or args.rope or args.qkv_epilogue or args.qkv_proj
               or args.layer_path or args.thin_pass or args.steady or args.contention)
    if special:
        if not torch.cuda.is_available():
            print("bench.py: no GPU visible", file=sys.stderr)
            return 2
        ob.load()
        if args.split:
            ob.oppo_set_option(ob.OPT_SPLIT_KV, args.split)
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
    if args.qkv_proj:
        return qkv_proj_bench(args, cfg, torch, ob)
    if args.layer_path:
        return layer_path_bench(args, cfg, torch, ob)
    if args.thin_pass:
        return thin_pass_bench(args, cfg, torch, ob)
    if args.steady:
        return steady_bench(args, cfg, torch, ob)
    if args.contention:
        return contention_study(args, cfg, torch, ob)
    if args.traffic_from:
        return traffic_from(args)
    if args.fp8_cache:
        return fp8_cache_bench(args, cfg, torch, ob)
    threads = min(16, len(os.sched_getaffinity(0)))
    ep = build_episode(cfg, threads=threads)
    # the oracle first: its process pool forks, which has to happen before this process touches the GPU
    baseline = None if args.no_cpu_baseline else cpu_baseline(cfg, ep)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    ob.load()
    if args.split:
        ob.oppo_set_option(ob.OPT_SPLIT_KV, args.split)
    head = measure_workload(cfg, ep, args, torch, ob, steps=args.steps, warmup=args.warmup, details=args.details)
    del ep
    line = {
        "metric": "chunked-prefill attn TFLOP/s + KV GB/s, % of MI355X roofline, 1 GPU",
        "value": head["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": head["config"],
    }
    for key in ("settle_ms", "kv_read_GBps", "total_GBps", "frac_of_roofline_episode", "frac_mfma_peak", "frac_hbm_peak",
                "prompt_prefill_ms", "roofline", "append_kernel_ms_per_step", "merge_kernel_ms_per_step", "step0",
                "pass_cold", "host_us_per_pass"):
        line[key] = head[key]
    per = {}
    if not args.single:
        for ci in sorted(CONFIGS):
            if ci == cfg.index:
                continue
            c = CONFIGS[ci]
            e = build_episode(c, threads=threads)
            if ci == 1:
                per["1"] = tiny_parity(c, e, torch, ob)
            else:
                r = measure_workload(c, e, args, torch, ob, steps=None, warmup=3, details="")
                rf = r["roofline"]
                per[str(ci)] = {"workload": r["config"]["workload"], "value": r["value"], "unit": "TFLOP/s",
                                "ms_per_step": r["ms_per_step"], "steps": r["steps"], "kv_read_GBps": r["kv_read_GBps"],
                                "total_GBps": r["total_GBps"], "bound": rf["bound"], "frac": rf["frac"],
                                "achieved": rf["achieved"], "achieved_unit": rf["unit"], "traffic": rf["traffic"],
                                "frac_of_roofline_episode": r["frac_of_roofline_episode"], "step0": r["step0"],
                                "pass_cold_value": r["pass_cold"]["value"], "merge_kernel_ms_per_step": r["merge_kernel_ms_per_step"],
                                "host_us_per_pass": r["host_us_per_pass"]}
            del e
            gc.collect()
            torch.cuda.empty_cache()
    line["per_config"] = per
    if not args.single:
        # the rows beyond the headline path, briefly, so that the default run shows them too: the small-chunk
        # workload through the cache of 8-bit codes (append + attention calls) and the fused QKV projection
        nxt = {}
        c3 = CONFIGS[3]
        e3 = build_episode(c3, threads=threads)
        keep = args.two_call
        args.two_call = True
        r8 = measure_workload(c3, e3, args, torch, ob, steps=None, warmup=3, fp8=True)
        args.two_call = keep
        del e3
        nxt["fp8_cache_config3"] = {"workload": r8["config"]["workload"], "step": r8["config"]["step"], "value": r8["value"], "unit": "TFLOP/s",
                                    "ms_per_step": r8["ms_per_step"], "steps": r8["steps"], "kv_read_GBps": r8["kv_read_GBps"],
                                    "total_GBps": r8["total_GBps"], "dtype": "fp8 (E4M3) cache, bf16 in / out",
                                    "roofline": {k: r8["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac", "kernel", "avg_launch_ms")},
                                    "episode_speedup_vs_16bit_cache_fused_step": (per["3"]["ms_per_step"] / r8["ms_per_step"]) if "3" in per else None}
        nxt["fp8_cache_config3"]["roofline"]["kernel"] = "attn_fwd_fp8_kernel"
        pr, wl, _, _ = qkv_proj_measure(args, cfg if cfg.head_dim == 128 else CONFIGS[2], torch, ob, only_fused=True)
        f = pr["fused_projection_rope_append"]
        nxt["qkv_proj"] = {"workload": wl, "value": f["tflops"], "unit": "TFLOP/s", "ms": f["ms"], "dtype": "bf16",
                           "roofline": {"bound": "mfma", "achieved": f["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                                        "frac": f["frac_of_mfma_peak"], "kernel": "qkv_proj_kernel"}}
        line["next_rows"] = nxt
    line["cpu_baseline"] = baseline
    print(json.dumps(line))
    return 0


def fp8_cache_bench(args, cfg, torch, ob) -> int:
    """The same workload through the 16-bit cache and through the 8-bit one (both as append + attention)."""
    from paper_2509_25762_amd.workload import build_episode
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    ob.load()
    ep = build_episode(cfg, threads=min(16, len(os.sched_getaffinity(0))))
    args.two_call = True
    out = {"metric": "chunked-prefill attention over a 16-bit and an 8-bit KV cache, 1 GPU", "n_gpus": 1, "data": "synthetic"}
    for name, fp8 in (("bf16_cache", False), ("fp8_cache", True)):
        r = measure_workload(cfg, ep, args, torch, ob, steps=None, warmup=3, fp8=fp8)
        out[name] = {k: r[k] for k in ("value", "ms_per_step", "steps", "kv_read_GBps", "total_GBps", "roofline",
                                       "append_kernel_ms_per_step", "merge_kernel_ms_per_step", "pass_cold", "config")}
    out["speedup_episode"] = out["bf16_cache"]["ms_per_step"] / out["fp8_cache"]["ms_per_step"]
    print(json.dumps(out))
    return 0


def tiny_parity(cfg, ep, torch, ob):
    """The tiny workload streamed through the library and compared, every row, with the float64
    oracle's one-shot prefill (tolerance of the parity tests); the cache bit for bit."""
    from oracle import bf16_bits_to_f64, full_prefill
    from paper_2509_25762_amd.episode import StreamedEpisode, uniform_chunks
    se = StreamedEpisode(ep, uniform_chunks(ep.prompt_len, ep.resp_len, cfg.chunk))
    se.run()
    torch.cuda.synchronize()
    got = bf16_bits_to_f64(se.scatter_outputs().cpu().numpy().view(np.uint16))
    worst, total, count, cache_ok = 0.0, 0.0, 0, True
    ck = se.cache_k.cpu().numpy().view(np.uint16)
    cv = se.cache_v.cpu().numpy().view(np.uint16)
    for i in range(cfg.batch):
        lo, hi = int(ep.tok_begin[i]), int(ep.tok_begin[i + 1])
        ref = full_prefill(bf16_bits_to_f64(ep.q[lo:hi]), bf16_bits_to_f64(ep.k[lo:hi]), bf16_bits_to_f64(ep.v[lo:hi]),
                           cfg.softmax_scale)
        err = np.abs(got[lo:hi] - ref)
        worst, total, count = max(worst, float(err.max())), total + float(err.sum()), count + err.size
        b = int(se.slot_begin[i])
        cache_ok = cache_ok and np.array_equal(ck[b:b + hi - lo], ep.k[lo:hi]) and np.array_equal(cv[b:b + hi - lo], ep.v[lo:hi])
    mean = total / max(1, count)
    return {"workload": f"config 1 ({cfg.name}): every row of the streamed episode against the float64 oracle",
            "parity": bool(worst <= 2e-2 and mean <= 2e-3 and cache_ok), "max_abs_err": worst, "mean_abs_err": mean,
            "cache_bit_exact": bool(cache_ok)}


def measure_workload(cfg, ep, args, torch, ob, steps, warmup, details="", fp8=False):
    """One workload through the timed protocol.  steps=None: as many episodes as fit ~0.25 s.
    fp8: through the cache of 8-bit codes (append + attention calls; scales = largest magnitude / 448)."""
    from paper_2509_25762_amd.episode import StreamedEpisode, StreamedEpisodeFp8, uniform_chunks
    from paper_2509_25762_amd.workload import episode_work
    chunks = uniform_chunks(ep.prompt_len, ep.resp_len, cfg.chunk)
    T = len(chunks) - 1
    if fp8:
        def amax(bits):
            return float(np.abs((bits.astype(np.uint32) << np.uint32(16)).view(np.float32)).max())
        ks, vs = amax(ep.k) / 448.0, amax(ep.v) / 448.0
        copies = [StreamedEpisodeFp8(ep, chunks, ks, vs, use_workspace=not args.no_workspace) for _ in range(max(1, args.copies))]
    else:
        copies = [StreamedEpisode(ep, chunks, use_workspace=not args.no_workspace) for _ in range(max(1, args.copies))]
    ncp = len(copies)
    # shared inputs are identical across copies; only the cache slabs and outputs differ
    work = episode_work(cfg, [(s.kv_before, s.q_len) for s in copies[0].steps[1:]])
    if fp8:
        for w in work:
            w["kv_read_bytes"] *= 0.5            # one byte per cached element
            w["append_bytes"] *= 0.75            # 16-bit rows in, 8-bit codes out
    flops = sum(w["flops"] for w in work)
    kv_bytes = sum(w["kv_read_bytes"] for w in work)
    tot_bytes = sum(w["kv_read_bytes"] + w["qo_bytes"] + w["append_bytes"] for w in work)
    fused = not args.two_call and not fp8
    peak_tflops = PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS

    # prompt prefill, once per copy, timed on its own
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for se in copies:
        se.reset(0)
        se.run_step(0)
    torch.cuda.synchronize()
    prompt_ms = (time.perf_counter() - t0) * 1e3 / ncp

    def episode(se):
        se.reset(1)
        for t in range(1, T + 1):
            se.run_step(t, fused=fused)

    def interleaved(k):
        """Episodes k*ncp .. k*ncp+ncp-1 pass by pass over the copies: between two passes of one copy
        every other copy's pass has run, so the copy's keys have left the last-level cache."""
        for se in copies:
            se.reset(1)
        for t in range(1, T + 1):
            for se in copies:
                se.run_step(t, fused=fused)

    def timed_region(run_one, n):
        """n calls of run_one(i) between two synchronisations; wall milliseconds per call."""
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            run_one(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / max(1, n)

    # (a full pass of Python's cyclic garbage collector takes tens of milliseconds of host time, during which
    # nothing is enqueued and the clocks fall back: it runs now, and not again until the timing is over)
    gc.collect()
    gc.disable()
    # warm-up as asked, then keep the GPU loaded until SETTLE_MS of work have run in all, right up to the
    # synchronisation that opens the timed region
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    done = 0
    settle_ms = 0.0
    batch = max(1, warmup)
    while True:
        ev0.record()
        for _ in range(batch):
            episode(copies[done % ncp])
            done += 1
        ev1.record()
        ev1.synchronize()
        got = ev0.elapsed_time(ev1)
        settle_ms += got
        if settle_ms >= SETTLE_MS:
            break
        batch = int(np.ceil((SETTLE_MS - settle_ms) / max(got / batch, 1e-3))) + 1
    est_ms = got / batch
    if steps is None:
        steps = int(min(400, max(8, np.ceil(250.0 / max(est_ms, 1e-3)))))

    ms_per_step = timed_region(lambda i: episode(copies[(done + i) % ncp]), steps)

    # the same episodes, interleaved pass by pass over the copies (every pass cold)
    n_groups = max(1, min(steps, 60) // ncp)
    cold_ms = timed_region(interleaved, n_groups) / ncp

    # kernel-level timing: the library brackets each of its kernel launches with HIP events on the
    # launch stream (the stream the kernels run on).  The episodes are enqueued back to back like the
    # timed ones and the events are read once at the end, so the kernels are timed at the clock rate
    # the sustained load settles at.  Host cost of the calls is collected in the same pass.
    prof_steps = int(min(steps, 50))
    ob.oppo_profile_enable(True)
    ob.oppo_profile_read()
    ob.oppo_profile_host()
    call_us = np.zeros(T)
    for s_ in range(prof_steps):
        episode(copies[s_ % ncp])
    each_ms, each_kind = ob.oppo_profile_read_each()
    ob.oppo_profile_host()
    # what a pass costs on the host: every call starts on an empty queue (synchronised first), so that the
    # time is the call's own and not the wait for room in a queue the host has filled
    call_us[:] = 0.0
    host_reps = 3
    for s_ in range(host_reps):
        se = copies[s_ % ncp]
        se.reset(1)
        for t in range(1, T + 1):
            torch.cuda.synchronize()
            h0 = time.perf_counter()
            se.run_step(t, fused=fused)
            call_us[t - 1] += (time.perf_counter() - h0) * 1e6 / host_reps
    host_us, host_calls = ob.oppo_profile_host()
    ob.oppo_profile_read()
    ob.oppo_profile_enable(False)
    gc.enable()
    attn_total_ms = float(each_ms[each_kind == 0].sum()) / prof_steps
    merge_total_ms = float(each_ms[each_kind == 1].sum()) / prof_steps
    append_total_ms = float(each_ms[each_kind == 2].sum()) / prof_steps
    launches_per_step = float(np.sum(each_kind == 0)) / prof_steps
    # per pass: launches come in call order, a pass = its attention launch(es), then its merge launch(es)
    pass_attn_ms = np.zeros(T)
    pass_merge_ms = np.zeros(T)
    per_pass_ok = False
    if fused:
        # walk the launch list: passes alternate attn+ [merge*]; the count of attention launches per pass is
        # the same in every episode, so the list splits evenly
        n_attn = int(np.sum(each_kind == 0))
        if n_attn == prof_steps * T:     # one attention launch per pass (no work list outgrew a launch)
            t_idx = -1
            for ms_, kd in zip(each_ms, each_kind):
                if kd == 0:
                    t_idx += 1
                    pass_attn_ms[t_idx % T] += ms_ / prof_steps
                elif kd == 1 and t_idx >= 0:
                    pass_merge_ms[t_idx % T] += ms_ / prof_steps
            per_pass_ok = True

    tflops = flops / (ms_per_step * 1e-3) / 1e12
    achieved = flops / (attn_total_ms * 1e-3) / 1e12
    # which roof binds the attention kernel on this workload (classical roofline over the episode's launches)
    bound = "mfma" if flops / (peak_tflops * 1e12) >= tot_bytes / (PEAK_HBM_GBPS * 1e9) else "hbm"
    achieved_gbps = tot_bytes / (attn_total_ms * 1e-3) / 1e9
    t_roof_ms = sum(max(w["flops"] / (peak_tflops * 1e12),
                        (w["kv_read_bytes"] + w["qo_bytes"] + w["append_bytes"]) / (PEAK_HBM_GBPS * 1e9)) for w in work) * 1e3
    traffic, traffic_note = (None, "no counter run on record for the 8-bit variant") if fp8 else measured_traffic(cfg.index)
    with_merge_ms = attn_total_ms + merge_total_ms
    res = {
        "value": tflops, "ms_per_step": ms_per_step, "steps": int(steps), "settle_ms": settle_ms,
        "config": {"workload": f"config {cfg.index} ({cfg.name}): B={cfg.batch}, Hq/Hkv/D={cfg.num_q_heads}/"
                               f"{cfg.num_kv_heads}/{cfg.head_dim}, C={cfg.chunk}, {T} passes per episode, "
                               f"{int(sum(w['rows'] for w in work))} response rows",
                   "step": ("one streamed episode (one oppo_chunk_step per pass: KV append + chunked-prefill attention)"
                            if fused else "one streamed episode (oppo_kv_append_fp8 + oppo_chunk_prefill_attn_fp8 per pass)"
                            if fp8 else "one streamed episode (oppo_kv_append + oppo_chunk_prefill_attn per pass)"),
                   "cache_copies_rotated": ncp},
        "kv_read_GBps": kv_bytes / (ms_per_step * 1e-3) / 1e9,
        "total_GBps": tot_bytes / (ms_per_step * 1e-3) / 1e9,
        "frac_of_roofline_episode": t_roof_ms / ms_per_step,
        "frac_mfma_peak": tflops / peak_tflops,
        "frac_hbm_peak": tot_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBPS,
        "prompt_prefill_ms": prompt_ms,
        "roofline": {"bound": bound, "achieved": achieved if bound == "mfma" else achieved_gbps,
                     "peak": peak_tflops if bound == "mfma" else PEAK_HBM_GBPS,
                     "unit": "TFLOP/s" if bound == "mfma" else "GB/s",
                     "frac": achieved / peak_tflops if bound == "mfma" else achieved_gbps / PEAK_HBM_GBPS,
                     "traffic": traffic, "traffic_note": traffic_note,
                     "algorithmic_bytes_per_launch": sum(w["kv_read_bytes"] + w["qo_bytes"] +
                                                         (w["append_bytes"] if fused else 0) for w in work) / T,
                     "kernel": "attn_fwd_kernel",
                     "launches_per_step": launches_per_step, "avg_launch_ms": attn_total_ms / max(launches_per_step, 1e-9),
                     # the same with the merge kernel's time in the denominator (the cost of the plan that was run)
                     "achieved_with_merge": (flops / (with_merge_ms * 1e-3) / 1e12) if bound == "mfma"
                                            else tot_bytes / (with_merge_ms * 1e-3) / 1e9,
                     "frac_with_merge": (flops / (with_merge_ms * 1e-3) / 1e12 / peak_tflops) if bound == "mfma"
                                        else tot_bytes / (with_merge_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS},
        "append_kernel_ms_per_step": append_total_ms,
        "merge_kernel_ms_per_step": merge_total_ms,
        "pass_cold": {"value": flops / (cold_ms * 1e-3) / 1e12, "unit": "TFLOP/s", "ms_per_step": cold_ms,
                      "kv_read_GBps": kv_bytes / (cold_ms * 1e-3) / 1e9,
                      "how": f"{ncp} episodes interleaved pass by pass over the cache copies"},
        "host_us_per_pass": {"library_plan": host_us["plan"] / max(1, host_calls), "library_launch": host_us["launch"] / max(1, host_calls),
                             "binding_call_wall": float(call_us.sum()) / T,
                             "kernel_us_per_pass": with_merge_ms * 1e3 / T},
    }
    w0 = work[0]
    if per_pass_ok:
        k0 = pass_attn_ms[0]
        b0 = w0["kv_read_bytes"] + w0["qo_bytes"] + w0["append_bytes"]
        res["step0"] = {"what": "the first response pass (full batch) on its own, attention kernel time",
                        "kernel_ms": k0, "tflops": w0["flops"] / (k0 * 1e-3) / 1e12, "total_GBps": b0 / (k0 * 1e-3) / 1e9,
                        "kv_read_GBps": w0["kv_read_bytes"] / (k0 * 1e-3) / 1e9,
                        "frac": (w0["flops"] / (k0 * 1e-3) / 1e12 / peak_tflops) if bound == "mfma"
                                else b0 / (k0 * 1e-3) / 1e9 / PEAK_HBM_GBPS}
        res["host_us_per_pass"]["binding_call_wall_by_pass"] = call_us.round(1).tolist()
        res["host_us_per_pass"]["kernel_us_by_pass"] = ((pass_attn_ms + pass_merge_ms) * 1e3).round(1).tolist()
    else:
        res["step0"] = None
    if details:
        det = {"attn_pass_ms": pass_attn_ms.tolist(), "merge_pass_ms": pass_merge_ms.tolist(), "work": work,
               "ms_per_step": ms_per_step, "call_us": call_us.tolist()}
        with open(details, "w") as f:
            json.dump(det, f, indent=1)
    del copies
    gc.collect()
    torch.cuda.empty_cache()
    return res


def traffic_from(args) -> int:
    """Turns the counter files of rocprofv3 --pmc FETCH_SIZE / --pmc WRITE_SIZE runs of this program into
    profiles/hbm_traffic.json.  --traffic-from takes a directory holding, per workload N, the csv outputs
    `cfgN_fetch*counter_collection.csv` and `cfgN_write*counter_collection.csv` of
        rocprofv3 --pmc FETCH_SIZE  ... -o cfgN_fetch -- python3 bench.py --config N --single --no-cpu-baseline --steps 12 --warmup 4
        rocprofv3 --pmc WRITE_SIZE  ... -o cfgN_write -- python3 bench.py --config N --single --no-cpu-baseline --steps 12 --warmup 4
    and, for the calibration, `cal_fetch*` / `cal_write*` of the same two commands with `--config 2 --two-call`
    (its append kernel is a plain copy of known size).  Counters are KiB per dispatch."""
    import csv
    import glob
    import subprocess
    from paper_2509_25762_amd.workload import CONFIGS, draw_lengths

    def per_kernel(pattern):
        files = sorted(glob.glob(os.path.join(args.traffic_from, "**", pattern), recursive=True))
        if not files:
            return None
        acc = {}
        for fn in files:
            with open(fn) as f:
                for row in csv.DictReader(f):
                    name = row.get("Kernel_Name", "")
                    val = float(row.get("Counter_Value", 0.0))
                    key = ("attn" if "attn_fwd_kernel" in name else "append" if "kv_append_kernel" in name else None)
                    if key:
                        acc.setdefault(key, []).append(val)
        return acc

    cal_f, cal_w = per_kernel("cal_fetch*counter_collection.csv"), per_kernel("cal_write*counter_collection.csv")
    if not cal_f or not cal_w or "append" not in cal_f or "append" not in cal_w:
        print("bench.py: calibration runs (cal_fetch*, cal_write*) not found", file=sys.stderr)
        return 2
    # the largest append launch is the full-batch pass: rows x Hkv x D x 2 bytes for K and again for V
    c2 = CONFIGS[2]
    P, R = draw_lengths(c2)
    rows0 = int(np.minimum(c2.chunk, R).sum())
    true_kib = 2.0 * rows0 * c2.num_kv_heads * c2.head_dim * 2 / 1024.0
    f_scale = true_kib / max(cal_f["append"])
    w_scale = true_kib / max(cal_w["append"])
    out = {"unit": "bytes per attn_fwd_kernel launch (HBM reads + writes), response-pass launches averaged",
           "method": "rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (KiB per dispatch), each scaled by what the same counter "
                     "reads for the append kernel of the full-batch pass of config 2 in a --two-call run (a plain copy of known size)",
           "fetch_scale": f_scale, "write_scale": w_scale, "source_fingerprint": source_fingerprint(), "configs": {}}
    try:
        out["commit"] = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True, text=True).stdout.strip() or "?"
    except OSError:
        out["commit"] = "?"
    for ci in sorted(CONFIGS):
        f, w = per_kernel(f"cfg{ci}_fetch*counter_collection.csv"), per_kernel(f"cfg{ci}_write*counter_collection.csv")
        if not f or not w or "attn" not in f or "attn" not in w:
            continue
        T = int(-(-int(draw_lengths(CONFIGS[ci])[1].max()) // CONFIGS[ci].chunk))
        # the first launches of a run are the prompt prefills (one per cache copy): drop them, keep whole episodes
        fa, wa = np.array(f["attn"][args.copies:]), np.array(w["attn"][args.copies:])
        fa, wa = fa[: len(fa) // T * T], wa[: len(wa) // T * T]
        out["configs"][str(ci)] = {"fetch_KiB": float(fa.mean()), "write_KiB": float(wa.mean()),
                                   "traffic_bytes_per_launch": float((fa.mean() * f_scale + wa.mean() * w_scale) * 1024.0),
                                   "launches_averaged": int(len(fa))}
    os.makedirs(os.path.dirname(TRAFFIC_FILE), exist_ok=True)
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
