#!/usr/bin/env python3
"""Benchmark of the on-GPU serving step on one MI355X.

A "step" is one iteration of the serving loop: scheduler step (retire, ring poll, FCFS admission, KV block
allocation, batch metadata), forward pass over paged KV (prefill or decode), sampling, publication.
The whole request set of the workload is resident in the HBM ring before the timed region starts
(saturation load). An untimed fill phase runs until the device has filled its batch and replaced one batch worth
of requests by later ones (steady state: prefill and decode iterations alternate as requests finish), then W
warm-up iterations run untimed, then
exactly K iterations are timed on the product path (one HIP graph launch per iteration); K further iterations
run with the dominant kernel's launches bracketed by HIP events for the roofline figure.

Prints ONE JSON line: output tokens/s over the timed iterations, p50/p99 inter-token latency from device
timestamps, scheduling microseconds per iteration, the HBM roofline of the dominant kernel, the whole decode and
prefill steps against their rooflines, the workload's own arrival process (open loop) isolated and under a host
memory-bandwidth stressor, the claim latency of an idle engine, and the CPU oracle's rate on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import synth  # noqa: E402

HBM_PEAK_GBS = 8000.0
PHASE_NAMES = {2: "k_qkv", 5: "k_oproj", 7: "k_gateup", 8: "k_down", 10: "k_lm_head", 4: "k_attention",
               16: "k_moe_router", 17: "k_moe_route", 18: "k_moe_gateup", 19: "k_moe_down", 20: "k_moe_combine"}

WORKLOADS = {
    "tiny": dict(model="tiny", workload="tiny", wseed=1000, rseed=2000, steps=30, warmup=3),
    "churn": dict(model="churn", workload="churn", wseed=1001, rseed=2001, steps=600, warmup=20),
    "llama3_8b": dict(model="llama3_8b", workload="llama3_8b", wseed=1002, rseed=2002, steps=200, warmup=60),
    "sched_stress": dict(model="sched_stress", workload="sched_stress", wseed=1003, rseed=2003, steps=100, warmup=5),
    # the mixture-of-experts model of the paper's evaluation (section 6) under the same request mix as the dense model
    "moe_30b_a3b": dict(model="moe_30b_a3b", workload="llama3_8b", wseed=1004, rseed=2002, steps=100, warmup=20),
}


def experts_hit(cfg, n_tokens):
    """Expected number of distinct experts that n_tokens tokens select under uniform routing (the synthetic router's):
    the experts whose matrices a grouped GEMM has to read."""
    E, k = cfg["n_experts"], cfg["n_active"]
    return E * (1.0 - (1.0 - k / E) ** n_tokens)


def phase_bytes(cfg, phase, n_tokens, n_seqs, ctx_tokens=0):
    """Algorithmic HBM bytes of one launch of a GEMM phase: the weight matrix once, plus the activations it reads
    and writes once (bf16 path: bf16 operands, fp32 residual stream read + written; fp32 path: fp32 throughout)."""
    bf = cfg["dtype"] == 1
    es, ea = (2, 2) if bf else (4, 4)
    d, F, V = cfg["d_model"], cfg["d_ffn"], cfg["vocab"]
    qkv_n = (cfg["n_q_heads"] + 2 * cfg["n_kv_heads"]) * cfg["head_dim"]
    no = cfg["n_q_heads"] * cfg["head_dim"]
    T, B = n_tokens, n_seqs
    if phase == 16:     # router: its matrix, the normalised x in, fp32 logits out
        return es * cfg["n_experts"] * d + T * (ea * d + 4 * cfg["n_experts"])
    if phase == 18:     # grouped gate/up: the matrices of the experts hit, x gathered per (token, expert) pair, the pairs' hidden rows out
        return es * 2 * F * d * experts_hit(cfg, T) + T * cfg["n_active"] * (ea * d + 2 * F)
    if phase == 19:     # grouped down: the matrices of the experts hit, the pairs' hidden rows in, fp32 outputs of the pairs out
        return es * d * F * experts_hit(cfg, T) + T * cfg["n_active"] * (2 * F + 4 * d)
    if phase == 2:      # in: normalised x; out: q, k, v
        return es * qkv_n * d + T * (ea * d + ea * qkv_n)
    if phase == 5:      # in: attention output; residual read + write; bf16 path also writes the next packed operand
        return es * d * no + T * (ea * no + 8 * d + (2 * d if bf else 0))
    if phase == 7:      # in: normalised x; out: silu(gate)*up (bf16 path) or gate and up (fp32 path)
        return es * 2 * F * d + T * (ea * d + (2 * F if bf else 8 * F))
    if phase == 8:
        return es * d * F + T * ((2 * F if bf else 8 * F) + 8 * d + (2 * d if bf else 0))
    if phase == 10:     # logits are fp32
        return es * V * d + B * (ea * d + 4 * V)
    if phase == 4:      # decode attention: K and V of every context token once, the queries, the output
        kv_tok = 2 * cfg["n_kv_heads"] * cfg["head_dim"] * es
        return kv_tok * ctx_tokens + T * 2 * ea * no
    raise ValueError(phase)


def decode_step_bytes(cfg, n_seqs, ctx_tokens):
    """Algorithmic HBM bytes of one decode iteration: every weight matrix once, the KV of every context
    token read once, one token of KV written per sequence, logits written and read by the sampler."""
    es = 2 if cfg["dtype"] == 1 else 4
    d, F, V, L = cfg["d_model"], cfg["d_ffn"], cfg["vocab"], cfg["n_layers"]
    qkv_n = (cfg["n_q_heads"] + 2 * cfg["n_kv_heads"]) * cfg["head_dim"]
    no = cfg["n_q_heads"] * cfg["head_dim"]
    if cfg.get("n_experts", 0):   # the router and the matrices of the experts this batch selects (expected count, uniform routing)
        ffn = cfg["n_experts"] * d + 3 * F * d * experts_hit(cfg, n_seqs)
    else:
        ffn = 3 * F * d
    w = es * (L * (qkv_n * d + d * no + ffn) + V * d)
    kv_tok = 2 * cfg["n_kv_heads"] * cfg["head_dim"] * es * L
    return w + kv_tok * (ctx_tokens + n_seqs) + 2 * 4 * n_seqs * V


def read_traffic(kernel, workload):
    """HBM bytes per launch from the committed counter summary (profiles/<kernel>_<workload>_hbm_traffic.md), or None."""
    path = os.path.join(ROOT, "profiles", "%s_%s_hbm_traffic.md" % (kernel, workload))
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_baseline(cfg, eng, raw, reqs, budget_tokens, n_req=4, prompt_cap=None):
    """The oracle, as it stands, on a bounded sample of the same workload."""
    from oracle import model as M, serve as SV
    sample = []
    for r in reqs[:n_req]:
        r = dict(r)
        r["max_new_tokens"] = min(r["max_new_tokens"], budget_tokens)
        if prompt_cap:
            r["prompt"] = r["prompt"][:prompt_cap]
        sample.append(r)
    # the oracle keeps its KV pool as dense fp64 arrays: size the pool to the sample, not to the engine's 64 GiB
    bs = eng["kv_block_size"]
    need = sum(max(1, -(-(len(r["prompt"]) + r["max_new_tokens"] - 1) // bs)) for r in sample)
    full_eng = eng
    eng = dict(eng, kv_num_blocks=need, max_batch=len(sample))
    t0 = time.perf_counter()
    ev, _ = SV.serve(cfg, M.Weights(cfg, raw), eng, sample)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    # the scheduler alone (integer state machine, single thread) over the whole request set with a constant token in
    # place of the model: the CPU figure that stands beside the on-GPU scheduling time per iteration
    from oracle import scheduler as SC
    sched = SC.Scheduler.from_engine(full_eng)
    t0 = time.perf_counter()
    sev = SV.run_schedule(sched, reqs, lambda plan: [1] * len(plan.sample_seq), max_iterations=400)
    sdt = time.perf_counter() - t0
    sched_us = 1e6 * sdt / max(1, sched.iteration)
    return dict(value=len(ev) / dt, unit="output tokens/s", cores=int(threads), kind="oracle",
                scheduler_only_us_per_iteration=round(sched_us, 1),
                scheduler_only_sample="%d iterations of the full request set, one thread, invariant checks included" % sched.iteration,
                sample="first %d requests, prompts %s(%s tokens), max_new_tokens capped at %d: %d output tokens in %.1f s"
                       % (len(sample), "truncated " if prompt_cap else "as drawn ", "+".join(str(len(r["prompt"])) for r in sample),
                          budget_tokens, len(ev), dt))


def _stress_worker(go, quit_, mib):
    """Host memory-bandwidth stressor: streaming copies between two buffers while `go` is set."""
    a = b = None
    while not quit_.is_set():
        if not go.wait(0.2):
            continue
        if a is None:
            a = np.ones(mib << 17, dtype=np.float64)
            b = np.empty_like(a)
        np.copyto(b, a)
        np.copyto(a, b)


class Stressor:
    """One streaming-copy process per host core (the synthetic stand-in for the paper's co-located tenants). The
    processes are started when the object is made (before this process touches the GPU) and idle until entered."""

    def __init__(self, n=None, mib=256):
        import multiprocessing as mp
        self.n = n or int(os.environ.get("OMP_NUM_THREADS", 0)) or os.cpu_count()
        ctx = mp.get_context("spawn")
        self.go, self.quit = ctx.Event(), ctx.Event()
        self.procs = [ctx.Process(target=_stress_worker, args=(self.go, self.quit, mib), daemon=True) for _ in range(self.n)]
        for p in self.procs:
            p.start()

    def __enter__(self):
        self.go.set()
        time.sleep(1.5)
        return self

    def __exit__(self, *a):
        self.go.clear()

    def close(self):
        self.go.clear()
        self.quit.set()
        for p in self.procs:
            p.join(timeout=10)
            if p.is_alive():
                p.terminate()


def open_loop(B, e, reqs, seconds):
    """The workload's own arrival process on an idle engine: a producer thread submits each request at its arrival time
    while the loop runs; the main thread polls. Returns TTFT (host clocks: submit -> first event seen) and ITL (device
    timestamps) percentiles and the output token rate over the run. Every request completes before it returns."""
    import threading
    reqs = [r for r in reqs if r["arrival_s"] <= seconds][: e.engine["ring_slots"] // 2]
    if not reqs:
        return None
    submit_t = {}
    e.set_exit_when_idle(False)
    e.run(0)
    t_start = time.perf_counter()

    def producer():
        for i, r in enumerate(reqs):
            dt = t_start + r["arrival_s"] - time.perf_counter()
            if dt > 0:
                time.sleep(dt)
            while True:
                try:
                    submit_t[e.submit_request(r)] = time.perf_counter()
                    break
                except B.BlinkError:
                    time.sleep(0.0005)

    th = threading.Thread(target=producer)
    th.start()
    evs, first_seen, done = [], {}, 0
    deadline = time.perf_counter() + seconds + 120
    while done < len(reqs) and time.perf_counter() < deadline:
        ev = e.poll(8192)
        now = time.perf_counter()
        if ev.size:
            evs.append(ev.copy())
            for rid in ev["request_id"][(ev["flags"] & 1) != 0]:
                first_seen[int(rid)] = now
            done += int(np.count_nonzero(ev["flags"] & 2))
        else:
            time.sleep(0.0002)
    t_end = time.perf_counter()
    th.join()
    e.stop()
    if done < len(reqs):
        raise RuntimeError("open loop: %d of %d requests completed" % (done, len(reqs)))
    ev = np.concatenate(evs)
    order = np.lexsort((ev["index"], ev["request_id"]))
    evs = ev[order]
    same = (evs["request_id"][1:] == evs["request_id"][:-1]) & (evs["index"][1:] == evs["index"][:-1] + 1)
    itl = (evs["device_ns"][1:].astype(np.int64) - evs["device_ns"][:-1].astype(np.int64))[same] / 1e6
    ttft = np.array([first_seen[r] - submit_t[r] for r in first_seen if r in submit_t]) * 1e3
    pct = lambda a, q: round(float(np.percentile(a, q)), 3) if len(a) else None
    return dict(requests=len(reqs), completed=done, seconds=round(t_end - t_start, 2), output_tokens=int(len(ev)),
                output_tokens_per_s=round(len(ev) / (t_end - t_start), 1),
                itl_ms=dict(p50=pct(itl, 50), p99=pct(itl, 99)), ttft_ms=dict(p50=pct(ttft, 50), p99=pct(ttft, 99)),
                arrivals="as drawn (producer thread stands in for the SmartNIC)")


def chunked_leg(B, cfg, eng, blob, reqs, K, W, args):
    """The same saturation run with chunked prefill (mixed prefill + decode iterations under the engine's token budget,
    the extension the paper names first): untimed fill until one batch worth of requests has been replaced by later ones,
    W warm-up iterations, K timed."""
    eng = dict(eng, chunked_prefill=True, max_prefill_tokens=max(args.chunk_budget, eng["max_batch"] + 1))
    e = B.Engine(cfg, eng, blob, flags=B.FLAG_TRACE | B.FLAG_EXIT_WHEN_IDLE | (B.FLAG_NO_GRAPH if args.no_graph else 0), trace_capacity=1 << 16,
                 tune=args.tune)
    ol = None
    try:
        if args.open_loop_seconds > 0:
            ol = open_loop(B, e, reqs, args.open_loop_seconds)     # the workload's own arrivals first (leaves the engine idle)
        e.set_exit_when_idle(True)
        for r in reqs:
            e.submit_request(r)
        base, fill = e.stats(), 0
        while fill < 4000:
            e.run(4)
            e.wait()
            e.drain(16384)
            st = e.stats()
            fill = int(st["iterations"] - base["iterations"])
            # steady: one batch worth of requests has been replaced by later ones (or everything has been admitted)
            if st["n_running"] == 0 or st["next_ticket"] - base["next_ticket"] >= min(len(reqs), 2 * eng["max_batch"]):
                break
        if W:
            e.run(W)
            e.wait()
        e.drain(16384)
        s0 = e.stats()
        t0 = time.perf_counter()
        e.run(K)
        e.wait()
        t1 = time.perf_counter()
        s1 = e.stats()
        ev = e.drain(16384)
        tr = e.trace(int(s1["iterations"] - s0["iterations"]))
        kernel_times = {}
        for ph in [int(x) for x in args.phases.split(",") if x]:
            sa = e.stats()
            e.time_phase(ph)
            e.run(K)
            e.wait()
            e.time_phase(-1)
            e.drain(16384)
            pms = e.phase_times_ms()
            n_it = min(len(pms), int(e.stats()["iterations"] - sa["iterations"]))
            n_l = 1 if ph in (0, 9, 10, 11) else cfg["n_layers"]
            if n_it:
                kernel_times[str(ph)] = round(1e3 * float(pms[:n_it].sum()) / (n_it * n_l), 2)
    finally:
        e.shutdown()
    iters = int(s1["iterations"] - s0["iterations"])
    ev = ev[ev["iteration"] >= s0["iterations"]]
    order = np.lexsort((ev["index"], ev["request_id"]))
    evs = ev[order]
    same = (evs["request_id"][1:] == evs["request_id"][:-1]) & (evs["index"][1:] == evs["index"][:-1] + 1)
    itl = (evs["device_ns"][1:].astype(np.int64) - evs["device_ns"][:-1].astype(np.int64))[same] / 1e6
    sched_us = (tr["t_sched_end_ns"].astype(np.int64) - tr["t_sched_begin_ns"].astype(np.int64)) / 1e3
    pct = lambda a, q: round(float(np.percentile(a, q)), 4) if len(a) else None
    d, F, V, L = cfg["d_model"], cfg["d_ffn"], cfg["vocab"], cfg["n_layers"]
    qkv_n = (cfg["n_q_heads"] + 2 * cfg["n_kv_heads"]) * cfg["head_dim"]
    layer_params = qkv_n * d + d * cfg["n_q_heads"] * cfg["head_dim"] + 3 * F * d
    toks_out = int(s1["tokens_out"] - s0["tokens_out"])
    flops = 2.0 * (L * layer_params * float(tr["n_tokens"].sum()) + V * d * toks_out)
    dt = t1 - t0
    return dict(value=round(toks_out / dt, 2), unit="output tokens/s", steps=iters, ms_per_step=round(1e3 * dt / max(1, iters), 4),
                token_budget_per_iteration=eng["max_prefill_tokens"], fill_iterations_before_warmup=fill,
                mean_tokens_per_iteration=round(float(tr["n_tokens"].mean()), 1) if len(tr) else None,
                mean_sequences_per_iteration=round(float(tr["n_seqs"].mean()), 1) if len(tr) else None,
                prompt_tokens_per_s=round(float(s1["tokens_prefilled"] - s0["tokens_prefilled"]) / dt, 1),
                projection_TFLOPs=round(flops / dt / 1e12, 1),
                frac_of_mfma_peak=round(flops / dt / 1e12 / (2500.0 if cfg["dtype"] == 1 else 157.3), 4),
                itl_ms=dict(p50=pct(itl, 50), p99=pct(itl, 99), n=int(len(itl))),
                sched_us_per_iteration=dict(median=pct(sched_us, 50), p99=pct(sched_us, 99)),
                **({"open_loop": ol} if ol else {}), **({"kernel_times_us": kernel_times} if kernel_times else {}))


def prefix_leg(B, cfg, eng, blob, reqs, args):
    """Prefix caching on a request set whose prompts start with common heads (system prompts): the whole set resident at
    t = 0 and run to completion, once without and once with the cache. Reports the time to serve the set, the prompt
    tokens computed, the blocks matched and evicted, and the scheduler's time per iteration (its table work is part of it)."""
    vocab = cfg["vocab"]
    lo, hi = [int(x) for x in args.prefix_len.split(",")]
    shared = synth.with_shared_prefixes(reqs, vocab, 77, n_prefixes=args.prefix_heads, prefix_len=(lo, hi), share=args.prefix_share)
    shared = [dict(r, prompt=r["prompt"][: eng["max_seq_len"] - r["max_new_tokens"]]) for r in shared]
    out = dict(workload="the workload's requests, %d %% of them behind one of %d common heads of %d..%d tokens"
                        % (round(100 * args.prefix_share), args.prefix_heads, lo, hi),
               requests=len(shared), prompt_tokens=int(sum(len(r["prompt"]) for r in shared)))
    for label, on in (("without_cache", False), ("with_cache", True)):
        e = B.Engine(cfg, dict(eng, prefix_cache=on), blob, flags=B.FLAG_TRACE | B.FLAG_EXIT_WHEN_IDLE, trace_capacity=1 << 16, tune=args.tune)
        try:
            for r in shared:
                e.submit_request(r)
            t0 = time.perf_counter()
            n_out = 0
            while True:
                e.run(64)
                e.wait()
                n_out += len(e.drain(1 << 16))
                st = e.stats()
                if st["n_running"] == 0 and st["next_ticket"] == len(shared):
                    break
            dt = time.perf_counter() - t0
            tr = e.trace(1 << 16)
        finally:
            e.shutdown()
        sched_us = (tr["t_sched_end_ns"].astype(np.int64) - tr["t_sched_begin_ns"].astype(np.int64)) / 1e3
        pre = tr["kind"] == 1
        out[label] = dict(seconds=round(dt, 2), output_tokens=n_out, output_tokens_per_s=round(n_out / dt, 1),
                          iterations=int(st["iterations"]), prefill_iterations=int(st["prefill_iterations"]),
                          prompt_tokens_computed=int(st["tokens_prefilled"]), blocks_matched=int(st["prefix_hit_blocks"]),
                          blocks_evicted=int(st["prefix_evictions"]),
                          sched_us=dict(median=round(float(np.median(sched_us)), 1), p99=round(float(np.percentile(sched_us, 99)), 1),
                                        max=round(float(sched_us.max()), 1),
                                        prefill_median=round(float(np.median(sched_us[pre])), 1) if pre.any() else None))
    a, b = out["without_cache"], out["with_cache"]
    out["speedup"] = round(a["seconds"] / b["seconds"], 3)
    out["prompt_tokens_saved_frac"] = round(1.0 - b["prompt_tokens_computed"] / max(1, a["prompt_tokens_computed"]), 3)
    return out


def cycle_weights(cfg, raw, period=16):
    """Weights of the same shapes whose greedy stream is known: attention output and FFN down projections zero (the
    residual stream stays the token's embedding) and row v of the LM head equal to the embedding of the token before v in
    its group of `period` consecutive ids, so that the largest logit after token t is that of t's successor in the group.
    Every stream then cycles with that period, and a lookup of its last two tokens finds the continuation: the input on
    which every draft is right."""
    V = cfg["vocab"]
    assert V % period == 0
    w = dict(raw)
    for l in range(cfg["n_layers"]):
        w[f"l{l}.wo"] = np.zeros_like(raw[f"l{l}.wo"])
        w[f"l{l}.wd"] = np.zeros_like(raw[f"l{l}.wd"])
    v = np.arange(V)
    w["lm"] = raw["embed"][(v // period) * period + (v % period - 1) % period]
    return w


def speculative_leg(B, cfg, eng, raw, reqs, args):
    """Speculative decoding on the workload's requests made greedy, the whole set resident at t = 0 and run to
    completion, without and with drafts, on two sets of weights. Random weights: a 32-layer random model neither copies
    from its context nor falls into a loop within a request's length, lookups find next to nothing, and the run shows
    what the draft kernel and the wider bookkeeping cost. Cycle weights (cycle_weights): every draft is right, the
    run shows what an iteration that verifies spec_tokens drafts per request costs against the tokens it saves: the
    upper bound of the gain at that draft count. Trained weights on text lie in between; there are none here."""
    greedy = [dict(r, temperature=0.0, top_k=0, top_p=1.0) for r in reqs]
    out = dict(workload="the workload's requests, greedy", requests=len(greedy), spec_tokens=args.spec_tokens)
    for wname in ("random_weights", "cycle_weights"):
        blob = synth.pack_blob(cfg, raw if wname == "random_weights" else cycle_weights(cfg, raw))
        res = {}
        for label, k in (("plain", 0), ("speculative", args.spec_tokens)):
            e = B.Engine(cfg, dict(eng, speculative=k), blob, flags=B.FLAG_TRACE | B.FLAG_EXIT_WHEN_IDLE, trace_capacity=1 << 16, tune=args.tune)
            try:
                for r in greedy:
                    e.submit_request(r)
                t0 = time.perf_counter()
                n_out = 0
                while True:
                    e.run(64)
                    e.wait()
                    n_out += len(e.drain(1 << 16))
                    st = e.stats()
                    if st["n_running"] == 0 and st["next_ticket"] == len(greedy):
                        break
                dt = time.perf_counter() - t0
                tr = e.trace(1 << 16)
            finally:
                e.shutdown()
            dec = tr[tr["kind"] == 2]
            dec_ms = (dec["t_publish_end_ns"].astype(np.int64) - dec["t_sched_begin_ns"].astype(np.int64)) / 1e6
            res[label] = dict(seconds=round(dt, 2), output_tokens=n_out, output_tokens_per_s=round(n_out / dt, 1),
                              iterations=int(st["iterations"]), prefill_iterations=int(st["prefill_iterations"]),
                              decode_iteration_ms_median=round(float(np.median(dec_ms)), 3) if len(dec) else None,
                              tokens_fed_per_decode_iteration=round(float(dec["n_tokens"].mean()), 1) if len(dec) else None,
                              decode_seconds=round(float(dec_ms.sum()) / 1e3, 2),
                              drafted=int(st["spec_drafted"]), accepted=int(st["spec_accepted"]))
        a, b = res["plain"], res["speculative"]
        res["speedup"] = round(a["seconds"] / b["seconds"], 3)
        res["decode_speedup"] = round(a["decode_seconds"] / max(1e-9, b["decode_seconds"]), 3)
        res["acceptance"] = round(b["accepted"] / max(1, b["drafted"]), 3)
        out[wname] = res
        del blob
    return out


def placement_leg(B, cfg, eng, blob, reqs, args, stressor):
    """Scheduler placement on one engine build (section 4.2 of the paper compares a GPU-resident with a CPU-resident
    scheduler on closed sets of N requests with I input and O output tokens at batch 16): N x I -> O sets, all resident
    at t = 0, served to completion by the device-decided loop and by the same engine with BLINK_FLAG_HOST_STEP (the
    launcher waits for every iteration, copies its tokens to the host and a batch description back, then enqueues the
    next one). Makespans, isolated and under the host stressor; sampling parameters as in the workload."""
    rng = np.random.default_rng(4242)
    sets = []
    for spec in args.placement_sets.split(","):
        n, i, o = [int(x) for x in spec.split("x")]
        sets.append((spec, [dict(reqs[j % len(reqs)], arrival_s=0.0, prompt=rng.integers(0, cfg["vocab"], i).astype(np.int32),
                                 max_new_tokens=o) for j in range(n)]))
    out = dict(sets="N x I x O: N requests of I prompt tokens and O output tokens (no end-of-sequence token), batch N",
               stressor=("%d processes, streaming copies of 2 x 256 MiB each" % stressor.n) if stressor else None)
    res = {spec: {} for spec, _ in sets}
    for label, flag in (("device_loop", 0), ("host_step", B.FLAG_HOST_STEP)):
        nmax = max(len(rs) for _, rs in sets)
        e = B.Engine(cfg, dict(eng, max_batch=max(nmax, 16), eos_token_id=-1), blob, flags=flag | B.FLAG_EXIT_WHEN_IDLE, tune=args.tune)
        try:
            def serve(rs):
                base = e.stats()["next_ticket"]
                for r in rs:
                    e.submit_request(r)
                want = sum(r["max_new_tokens"] for r in rs)
                t0 = time.perf_counter()
                e.run(0)
                n_out = 0
                while n_out < want and time.perf_counter() - t0 < 120:      # makespan: until the last token has been polled
                    n_out += len(e.poll(8192))
                dt = time.perf_counter() - t0
                e.wait()                                                    # (the iterations enqueued ahead run empty, untimed)
                n_out += len(e.drain(1 << 16))
                st = e.stats()
                if n_out != want or st["n_running"] != 0 or st["next_ticket"] != base + len(rs):
                    raise RuntimeError("placement leg: %d of %d tokens" % (n_out, want))
                return dt, n_out
            for spec, rs in sets:
                serve(rs[:2])                                  # warm: first launches, clocks
                dt, n_out = serve(rs)
                row = dict(seconds=round(dt, 4), output_tokens=n_out)
                if stressor:
                    with stressor:
                        dts, _ = serve(rs)
                    row["seconds_stressed"] = round(dts, 4)
                res[spec][label] = row
        finally:
            e.shutdown()
    for spec in res:
        a, b = res[spec]["device_loop"], res[spec]["host_step"]
        res[spec]["host_step_over_device_loop"] = round(b["seconds"] / a["seconds"], 4)
        if stressor:
            res[spec]["host_step_over_device_loop_stressed"] = round(b["seconds_stressed"] / a["seconds_stressed"], 4)
            res[spec]["stressed_over_isolated"] = dict(device_loop=round(a["seconds_stressed"] / a["seconds"], 4),
                                                       host_step=round(b["seconds_stressed"] / b["seconds"], 4))
    out["results"] = res
    return out


def claim_latency(B, e, vocab, n=24):
    """An idle engine (its scheduler kernel polling the ring on the device) receives one short request at a time:
    time from the entry of blink_submit, and from its return, to the end of the scheduler step that admitted the request
    (device clock, mapped to the host's monotonic clock by blink_clock_sync), beside the duration of the submit call."""
    rng = np.random.default_rng(7)
    e.set_exit_when_idle(False)
    e.run(0)
    rows = []
    try:
        time.sleep(0.05)
        for i in range(n):
            prompt = rng.integers(0, vocab, 8).astype(np.int32)
            t0 = time.clock_gettime_ns(time.CLOCK_MONOTONIC)
            rid = e.submit(prompt, 1)
            t1 = time.clock_gettime_ns(time.CLOCK_MONOTONIC)
            deadline = time.perf_counter() + 10
            while time.perf_counter() < deadline:
                ev = e.poll(64)
                if ev.size and np.any((ev["request_id"] == rid) & ((ev["flags"] & 2) != 0)):
                    break
                time.sleep(0.0005)
            dev, host, unc = e.clock_sync()
            rows.append((rid, t0, t1, dev - host, unc))
            time.sleep(0.02)
    finally:
        e.stop()
    tr = e.trace()
    adm = {}
    for t in tr:
        for k in range(int(t["n_admitted"])):
            adm[int(t["first_admitted"]) + k] = int(t["t_sched_end_ns"])
    entry, ret, call, unc = [], [], [], []
    for rid, t0, t1, off, u in rows:
        if rid in adm:
            claimed_host = adm[rid] - off
            entry.append((claimed_host - t0) / 1e3)
            ret.append((claimed_host - t1) / 1e3)
            call.append((t1 - t0) / 1e3)
            unc.append(u / 1e3)
    if not entry:
        return None
    med = lambda a: round(float(np.median(a)), 1)
    return dict(requests=len(entry), submit_call_us=med(call), submit_entry_to_scheduled_us=dict(median=med(entry), p90=round(float(np.percentile(entry, 90)), 1)),
                submit_return_to_scheduled_us=dict(median=med(ret), p90=round(float(np.percentile(ret, 90)), 1)),
                clock_mapping_uncertainty_us=med(unc),
                note="idle engine, one 8-token request at a time; 'scheduled' = end of the scheduler step that admitted it (claim, block "
                     "allocation and batch metadata done); blink_submit is two synchronous copies (payload, then the state word), so the "
                     "device may claim the request before the call returns")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0)
    ap.add_argument("--warmup", type=int, default=-1)
    ap.add_argument("--workload", default=os.environ.get("BLINK_BENCH_WORKLOAD", "llama3_8b"), choices=sorted(WORKLOADS))
    ap.add_argument("--phase", type=int, default=-1,
                    help="forward phase whose kernel is timed for the roofline (default: the dominant one of the workload: "
                         "decode attention for llama3_8b at its batch of 256, the gate/up GEMM otherwise)")
    ap.add_argument("--phases", default="", help="comma-separated forward phases (see blink_time_phase): after the roofline window, "
                    "--steps more iterations per phase with that phase's launches bracketed by HIP events; reports the average "
                    "launch duration in decode and in prefill iterations as kernel_times_us")
    ap.add_argument("--no-graph", action="store_true", help="enqueue the kernels one by one in every window (BLINK_FLAG_NO_GRAPH)")
    ap.add_argument("--tune", type=lambda x: int(x, 0), default=0, help="blink_config.tune")
    ap.add_argument("--preemption", action="store_true", help="on-demand KV growth with preemption instead of worst-case reservations "
                    "(BLINK_FLAG_PREEMPTION; the chunked-prefill leg is skipped)")
    ap.add_argument("--layers", type=int, default=0, help="tuning: build the model with this many layers instead of its own "
                    "(reported in config; not the workload's model any more)")
    ap.add_argument("--requests", type=int, default=0)
    ap.add_argument("--max-batch", type=int, default=0, help="override the engine's batch slots")
    ap.add_argument("--kv-blocks", type=int, default=0, help="override the size of the KV pool (16-token blocks)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-chunked-leg", action="store_true", help="skip the second saturation run with chunked prefill")
    ap.add_argument("--chunk-budget", type=int, default=2048, help="tokens per iteration of the run with chunked prefill")
    ap.add_argument("--only-chunked-leg", action="store_true", help="tuning: skip everything else")
    ap.add_argument("--prefix-leg", action="store_true", help="only this: the request set behind common prompt heads, served to "
                    "completion without and with prefix caching (BLINK_FLAG_PREFIX_CACHE)")
    ap.add_argument("--spec-leg", action="store_true", help="only this: the request set made greedy with repetitive prompts, served to "
                    "completion without and with speculative decoding")
    ap.add_argument("--placement-leg", action="store_true", help="only this: closed sets of N requests served by the device-decided "
                    "loop and by the same engine with a host round trip per iteration (BLINK_FLAG_HOST_STEP), isolated and "
                    "under the host stressor")
    ap.add_argument("--placement-sets", default="16x128x256,16x512x128,64x128x128", help="N x I x O sets of --placement-leg")
    ap.add_argument("--spec-tokens", type=int, default=4, help="most drafts per request and iteration in --spec-leg")
    ap.add_argument("--prefix-heads", type=int, default=8)
    ap.add_argument("--prefix-len", default="256,1024", help="range of the common heads' lengths in tokens")
    ap.add_argument("--prefix-share", type=float, default=0.8, help="fraction of the requests that start with a common head")
    ap.add_argument("--dump-iterations", default="",
                    help="write one line per iteration of the warm-up and the timed window (kind, sequences, tokens, context "
                         "tokens, timed flag): lets a rocprofv3 trace of the same run be split by iteration kind")
    ap.add_argument("--open-loop-seconds", type=float, default=8.0, help="0: skip the run with the workload's own arrivals")
    ap.add_argument("--rates", default="", help="comma-separated arrival rates (requests/s): one more open-loop run at each, "
                    "with the workload's lengths and arrival times redrawn at that rate")
    ap.add_argument("--interference", dest="interference", action="store_true", default=None,
                    help="repeat the open-loop run with a host memory-bandwidth stressor on every core and report the ratios "
                         "(default: on for llama3_8b)")
    ap.add_argument("--no-interference", dest="interference", action="store_false")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; one engine serves one GPU and nothing is sharded (--gpus 1 only)", file=sys.stderr)
        sys.exit(2)
    if args.interference is None:
        args.interference = args.workload == "llama3_8b"
    if args.workload == "moe_30b_a3b":
        args.no_chunked_leg = True
    stressor = Stressor() if ((args.interference and args.open_loop_seconds > 0) or args.placement_leg) else None   # before the GPU is touched
    import paper_2604_07609_amd as B

    if args.phase < 0:
        args.phase = 18 if args.workload == "moe_30b_a3b" else 4 if args.workload == "llama3_8b" and not args.max_batch else 7
    wl = WORKLOADS[args.workload]
    K = args.steps or wl["steps"]
    W = args.warmup if args.warmup >= 0 else wl["warmup"]
    cfg, eng = synth.model_config(wl["model"]), synth.engine_config(wl["model"])
    if args.layers:
        cfg["n_layers"] = args.layers
    t_gen = time.perf_counter()
    raw = synth.make_weights(cfg, wl["wseed"], threads=min(16, os.cpu_count() or 8))
    reqs = synth.make_workload(wl["workload"], cfg["vocab"], wl["rseed"], n_requests=args.requests or None)
    if args.max_batch:
        eng["max_batch"] = args.max_batch
    if args.kv_blocks:
        eng["kv_num_blocks"] = args.kv_blocks
    if args.preemption:
        eng["preemption"] = True
        args.no_chunked_leg = True
    reqs = reqs[: eng["ring_slots"]]
    blob = synth.pack_blob(cfg, raw)
    t_gen = time.perf_counter() - t_gen

    if args.prefix_leg:
        print(json.dumps(dict(prefix_cache=prefix_leg(B, cfg, eng, blob, reqs, args), config={"workload": args.workload, "requests": len(reqs)})))
        return
    if args.placement_leg:
        try:
            print(json.dumps(dict(scheduler_placement=placement_leg(B, cfg, eng, blob, reqs, args, stressor),
                                  config={"workload": args.workload, "layers": cfg["n_layers"]})))
        finally:
            stressor.close()
        return
    if args.spec_leg:
        print(json.dumps(dict(speculative=speculative_leg(B, cfg, eng, raw, reqs, args), config={"workload": args.workload, "requests": len(reqs)})))
        return
    if args.only_chunked_leg:
        print(json.dumps(chunked_leg(B, cfg, eng, blob, reqs, K, W, args)))
        return
    # One engine serves every leg. First the legs that leave it idle again (claim latency, the workload's own arrivals,
    # isolated and under the host stressor), then the saturation run that is timed.
    e = B.Engine(cfg, eng, blob, flags=B.FLAG_TRACE | (B.FLAG_NO_GRAPH if args.no_graph else 0), trace_capacity=1 << 18, tune=args.tune)
    claim = iso = stressed = stress_n = None
    sweep = []
    try:
        if args.open_loop_seconds > 0:
            claim = claim_latency(B, e, cfg["vocab"])
            iso = open_loop(B, e, reqs, args.open_loop_seconds)
            if stressor and iso:
                with stressor as st:
                    stressed = open_loop(B, e, reqs, args.open_loop_seconds)
                    stress_n = st.n
            for rate in [float(x) for x in args.rates.split(",") if x]:
                rr = synth.make_workload(wl["workload"], cfg["vocab"], wl["rseed"], n_requests=args.requests or None, rate=rate)
                res = open_loop(B, e, rr, args.open_loop_seconds)
                if res:
                    sweep.append(dict(rate_req_per_s=rate, **res))
        # ---- saturation: the whole request set resident in the ring ----
        e.set_exit_when_idle(True)
        sat0 = e.stats()
        for r in reqs:
            e.submit_request(r)
        # untimed fill, decided from device state: until the batch has filled (admission is strict FCFS and a decode
        # iteration only runs when nothing more can be admitted, so a decode iteration in the trace means the batch is as
        # full as batch slots and KV pool allow) AND one batch worth of requests has been replaced by later ones (the
        # first cohort starts together and finishes nothing for a while: timed straight after the fill, a short window
        # would see almost only decode iterations), or everything has been admitted
        fill, turn = 0, min(len(reqs), 2 * eng["max_batch"])
        seen_decode = False
        while fill < 20000:
            e.run(8)
            e.wait()
            e.drain(16384)
            st = e.stats()
            fill = int(st["iterations"] - sat0["iterations"])
            seen_decode = seen_decode or bool(np.any(e.trace(8)["kind"] == 2))
            if st["n_running"] == 0 or (seen_decode and st["next_ticket"] - sat0["next_ticket"] >= turn):
                break
        if W:
            e.run(W)
            e.wait()
        e.drain(16384)
        s0 = e.stats()
        t0 = time.perf_counter()
        e.run(K)                       # the timed window: K iterations on the product path (one graph launch per iteration)
        e.wait()                       # joins the launcher, which synchronises the compute stream
        t1 = time.perf_counter()
        s1 = e.stats()
        ev = e.drain(16384)
        # the same number of iterations again with the timed kernel's launches bracketed by HIP events on the compute
        # stream (kernels enqueued one by one instead of through the graph): the per-launch durations of the roofline
        e.time_phase(args.phase)
        e.run(K)
        e.wait()
        s2 = e.stats()
        e.time_phase(-1)
        e.drain(16384)
        phase_ms = e.phase_times_ms()
        kernel_times = {}
        for ph in [int(x) for x in args.phases.split(",") if x]:
            sa = e.stats()
            e.time_phase(ph)
            e.run(K)
            e.wait()
            e.time_phase(-1)
            e.drain(16384)
            sb = e.stats()
            pms = e.phase_times_ms()
            trx = e.trace(int(sb["iterations"] - sa["iterations"]))[: len(pms)]
            n_l = 1 if ph in (0, 9, 10, 11) else cfg["n_layers"]
            row = {}
            for label, kind in (("decode", 2), ("prefill", 1)):
                sel = trx["kind"] == kind
                if sel.any():
                    row[label] = round(1e3 * float(pms[: len(trx)][sel].sum()) / (int(sel.sum()) * n_l), 2)
            kernel_times[str(ph)] = row
        trace = e.trace(1 << 18)
        e.calibration_copy(64 << 20)    # one plain copy kernel of known size: scales the HBM counters of a --pmc run
        copy_gbs, mfma_tflops, read_gbs = e.calibration_rates()
    finally:
        e.shutdown()
        if stressor:
            stressor.close()
    chunked = None
    if not args.no_chunked_leg and eng["max_prefill_tokens"] > eng["max_batch"]:
        chunked = chunked_leg(B, cfg, eng, blob, reqs, K, W, args)

    if args.dump_iterations:
        with open(args.dump_iterations, "w") as f:
            f.write("# iteration kind n_seqs n_tokens ctx_tokens timed(1: timed window, 2: window with HIP events around the timed kernel) chain\n")
            for t in trace[trace["iteration"] < s2["iterations"]]:
                flag = 1 if s0["iterations"] <= t["iteration"] < s1["iterations"] else (2 if t["iteration"] >= s1["iterations"] else 0)
                f.write("%d %d %d %d %d %d %d\n" % (t["iteration"], t["kind"], t["n_seqs"], t["n_tokens"], t["ctx_tokens"], flag, t["chain"]))
    iters = int(s1["iterations"] - s0["iterations"])
    toks = int(s1["tokens_out"] - s0["tokens_out"])
    dt = t1 - t0
    tr = trace[(trace["iteration"] >= s0["iterations"]) & (trace["iteration"] < s1["iterations"])]
    # inter-token latency from device timestamps of consecutive tokens of a request, both inside the timed region
    itl = []
    ev = ev[ev["iteration"] >= s0["iterations"]]
    order = np.lexsort((ev["index"], ev["request_id"]))
    evs = ev[order]
    same = (evs["request_id"][1:] == evs["request_id"][:-1]) & (evs["index"][1:] == evs["index"][:-1] + 1)
    itl = (evs["device_ns"][1:].astype(np.int64) - evs["device_ns"][:-1].astype(np.int64))[same] / 1e6
    sched_us = (tr["t_sched_end_ns"].astype(np.int64) - tr["t_sched_begin_ns"].astype(np.int64)) / 1e3
    dec = tr["kind"] == 2
    # Roofline of the timed kernel. Its launches in decode iterations stream the weight matrix once (HBM bound); its
    # launches in prefill iterations are compute bound and are reported beside them against the MFMA peak.
    per_layer = 1 if args.phase in (10,) else cfg["n_layers"]
    trp = trace[(trace["iteration"] >= s1["iterations"]) & (trace["iteration"] < s2["iterations"])]   # the window with HIP events
    pm = phase_ms[: len(trp)]
    trp = trp[: len(pm)]
    decp = trp["kind"] == 2

    def klass(sel):
        n = int(sel.sum()) * per_layer
        if n == 0:
            return None
        ms = float(pm[sel].sum())
        by = float(sum(phase_bytes(cfg, args.phase, int(t["n_tokens"]), int(t["n_seqs"]), int(t["ctx_tokens"])) for t in trp[sel])) * per_layer
        return dict(launches=n, avg_launch_us=round(1e3 * ms / n, 3), bytes_per_launch=round(by / n), GBs=round(by / (ms * 1e-3) / 1e9, 2))

    d_cls, p_cls, a_cls = klass(decp), klass(~decp), klass(np.ones(len(pm), dtype=bool))
    kname = PHASE_NAMES.get(args.phase, str(args.phase))
    traffic = read_traffic(kname, args.workload)
    roofline = dict(bound="hbm", kernel=kname,
                    launch_class="launches of decode iterations" + (" (paged KV of every context read once)" if args.phase == 4 else " (weights read once)"),
                    achieved=d_cls["GBs"] if d_cls else None, peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(d_cls["GBs"] / HBM_PEAK_GBS, 4) if d_cls else None, traffic=traffic,
                    launches=d_cls["launches"] if d_cls else 0, avg_launch_us=d_cls["avg_launch_us"] if d_cls else None,
                    algorithmic_bytes_per_launch=d_cls["bytes_per_launch"] if d_cls else None,
                    all_launches=a_cls,
                    window="the %d iterations that follow the timed ones: same kernels enqueued one by one, the timed kernel's "
                           "launches bracketed by HIP events on the compute stream" % len(pm))
    if p_cls and args.phase != 4:
        es = 2 if cfg["dtype"] == 1 else 4
        if args.phase in (18, 19):    # grouped GEMMs: every (token, expert) pair meets one expert's matrices
            wbytes = es * (2 if args.phase == 18 else 1) * cfg["d_ffn"] * cfg["d_model"] * cfg["n_active"]
        else:
            wbytes = phase_bytes(cfg, args.phase, 0, 0)
        cols = "n_seqs" if args.phase == 10 else "n_tokens"     # the LM head runs on the last token of every sequence
        flops = float(sum(2.0 * (wbytes / es) * int(t[cols]) for t in trp[~decp])) * per_layer
        p_cls["TFLOPs"] = round(flops / (float(pm[~decp].sum()) * 1e-3) / 1e12, 1)
        p_cls["mfma_peak_TFLOPs"] = 2500.0 if cfg["dtype"] == 1 else 157.3
        roofline["prefill_launches"] = p_cls
    # whole-step view of the decode iterations: algorithmic bytes of the step over its duration on the device clock
    step_ns = np.diff(tr["t_sched_begin_ns"].astype(np.int64))
    dec_step = None
    if dec[:-1].sum() >= 1:
        idx = np.nonzero(dec[:-1])[0]
        b = np.array([decode_step_bytes(cfg, int(tr["n_seqs"][i]), int(tr["ctx_tokens"][i])) for i in idx], dtype=np.float64)
        gbs = float(b.sum() / step_ns[idx].sum())
        dec_step = dict(median_us=round(float(np.median(step_ns[idx])) / 1e3, 2), algorithmic_GBs=round(gbs, 2),
                        frac_of_hbm_peak=round(gbs / HBM_PEAK_GBS, 4), mean_batch=round(float(tr["n_seqs"][idx].mean()), 2),
                        mean_context_tokens=round(float(tr["ctx_tokens"][idx].mean() / max(1.0, tr["n_seqs"][idx].mean())), 1))
    # whole-step view of the prefill iterations: flops of the dense projections (2 x weights x tokens; the LM head on
    # the last token of every sequence; the causal attention products are left out, so this is a lower bound) over
    # the iterations' duration on the device clock, against the MFMA peak of the arithmetic type
    pre_step = None
    pre = tr["kind"] == 1
    if pre[:-1].sum() > 0:
        idx = np.nonzero(pre[:-1])[0]
        d, F, V, L = cfg["d_model"], cfg["d_ffn"], cfg["vocab"], cfg["n_layers"]
        qkv_n = (cfg["n_q_heads"] + 2 * cfg["n_kv_heads"]) * cfg["head_dim"]
        ffn_active = cfg["n_experts"] * d + cfg["n_active"] * 3 * F * d if cfg.get("n_experts", 0) else 3 * F * d
        layer_params = qkv_n * d + d * cfg["n_q_heads"] * cfg["head_dim"] + ffn_active
        fl = float(sum(2.0 * (L * layer_params * int(tr["n_tokens"][i]) + V * d * int(tr["n_seqs"][i])) for i in idx))
        secs = float(step_ns[idx].sum()) * 1e-9
        peak = 2500.0 if cfg["dtype"] == 1 else 157.3
        pre_step = dict(iterations=int(len(idx)), mean_tokens=round(float(tr["n_tokens"][idx].mean()), 1),
                        prompt_tokens_per_s=round(float(tr["n_tokens"][idx].sum()) / secs, 1),
                        projection_TFLOPs=round(fl / secs / 1e12, 1), mfma_peak_TFLOPs=peak,
                        frac_of_mfma_peak=round(fl / secs / 1e12 / peak, 4))
    out = {
        "metric": "output tokens/sec at 1 GPU; p50/p99 ITL; on-GPU scheduling us/iteration",
        "value": round(toks / dt, 2), "unit": "output tokens/s", "n_gpus": 1, "steps": iters, "warmup": W,
        "ms_per_step": round(1e3 * dt / max(1, iters), 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg["dtype"] == 1 else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "layers": cfg["n_layers"], "requests_resident": len(reqs), "arrivals": "all resident at t=0 (saturation)",
                   "max_batch": eng["max_batch"], "kv_blocks": eng["kv_num_blocks"],
                   "fill_iterations_before_warmup": fill, "preemption": bool(eng.get("preemption", False)),
                   "arithmetic": ("bf16 weights and KV cache; projections on the half-precision matrix-core path (weights re-encoded "
                                  "exactly, activations between GEMMs in half precision), attention products in bf16, fp32 accumulation")
                                 if cfg["dtype"] == 1 else "fp32",
                   "loop": "device-decided kernel chain, one HIP graph per iteration; host calls per iteration: 1 graph launch + 1 event "
                           "record by the launcher thread (it reads no result the device waits for)"},
        "itl_ms": {"p50": round(float(np.percentile(itl, 50)), 4) if len(itl) else None,
                   "p99": round(float(np.percentile(itl, 99)), 4) if len(itl) else None, "n": int(len(itl))},
        "sched_us_per_iteration": {"median": round(float(np.median(sched_us)), 2) if len(sched_us) else None,
                                   "p99": round(float(np.percentile(sched_us, 99)), 2) if len(sched_us) else None},
        "iterations": {"prefill": int((tr["kind"] == 1).sum()), "decode": int(dec.sum()),
                       "prefill_tokens": int(s1["tokens_prefilled"] - s0["tokens_prefilled"])},
        "decode_step": dec_step,
        "prefill_step": pre_step,
        "roofline": roofline,
        "measured_ceilings": {"copy_kernel_GBs": round(copy_gbs, 1), "read_kernel_GBs": round(read_gbs, 1), "mfma_bf16_loop_TFLOPs": round(mfma_tflops, 1),
                              "note": "plain kernels on this device: a 1 GiB copy (read + written), a 1 GiB read and a register-only MFMA loop"},
        "setup_s": {"weights_and_workload": round(t_gen, 1)},
    }
    if kernel_times:
        out["kernel_times_us"] = dict(kernel_times, note="average launch duration by phase number (blink_time_phase), HIP events, "
                                      "in the decode and the prefill iterations of a window of its own")
    if int(dec.sum()) == 0 and args.workload in ("llama3_8b", "churn"):
        out["warning"] = "the timed window holds no decode iteration"
        print("bench.py: the timed window holds no decode iteration (steps=%d): ITL and the decode roofline are empty" % K, file=sys.stderr)
    if chunked:
        out["chunked_prefill"] = chunked
    if claim:
        out["claim_latency"] = claim
    if iso:
        out["open_loop"] = iso
    if stressed:
        ratio = lambda a, b: round(a / b, 3) if a and b else None
        out["interference"] = dict(stressor="%d processes, streaming copies of 2 x 256 MiB each" % stress_n, stressed=stressed,
                                   ratio_stressed_over_isolated=dict(
                                       itl_p50=ratio(stressed["itl_ms"]["p50"], iso["itl_ms"]["p50"]),
                                       itl_p99=ratio(stressed["itl_ms"]["p99"], iso["itl_ms"]["p99"]),
                                       ttft_p50=ratio(stressed["ttft_ms"]["p50"], iso["ttft_ms"]["p50"]),
                                       ttft_p99=ratio(stressed["ttft_ms"]["p99"], iso["ttft_ms"]["p99"]),
                                       output_tokens_per_s=ratio(stressed["output_tokens_per_s"], iso["output_tokens_per_s"])))
    if sweep:
        out["open_loop_sweep"] = sweep
    del blob
    if not args.no_cpu_baseline:
        budget = args.cpu_sample_tokens or {"tiny": 32, "churn": 16, "llama3_8b": 4, "sched_stress": 16, "moe_30b_a3b": 4}[args.workload]
        if args.workload == "moe_30b_a3b":
            # the oracle widens every tensor it touches to fp64 and keeps it: all layers' experts would take 8 bytes x 29 G
            # parameters of host memory. It runs the model cut to its first layers (same embedding and LM head), and the
            # rate is scaled by the layer ratio (the layers dominate its time)
            keep = min(4, cfg["n_layers"])
            cut = dict(cfg, n_layers=keep)
            cb = cpu_baseline(cut, eng, raw, reqs, budget, n_req=2, prompt_cap=32)
            cb["value"] *= keep / cfg["n_layers"]
            cb["sample"] += "; model cut to its first %d of %d layers, rate scaled by %d/%d" % (keep, cfg["n_layers"], keep, cfg["n_layers"])
            out["cpu_baseline"] = cb
        elif args.workload == "llama3_8b":
            out["cpu_baseline"] = cpu_baseline(cfg, eng, raw, reqs, budget, n_req=2, prompt_cap=32)
        else:
            out["cpu_baseline"] = cpu_baseline(cfg, eng, raw, reqs, budget)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
