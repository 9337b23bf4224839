"""Parity at the full size of the benchmark: the llama3_8b-shaped model (32 layers, d 4096, 32 q / 8 kv heads of
128, FFN 14336, vocabulary 128256, bf16) in the engine configuration bench.py times (256 batch slots, 32768 KV
blocks, 8192 prefill tokens per iteration), on prompts drawn like the benchmark's (up to 4096 tokens).

The oracle cannot run such a batch (one forward pass over the fp64 weights takes seconds per token block), so
- the scheduler side is checked in full: batch metadata, block tables and the free stack of every iteration are
  bit-exact against the oracle's scheduler;
- the model side is checked on sampled outputs: the first two requests are short probes (16 tokens) that ride in
  the same iterations as the long prompts (prefill iterations of up to 8192 tokens through the tile kernels, decode
  iterations of 82 sequences). The oracle serves the two probes alone, teacher-forced with the engine's tokens; a
  request's logits do not depend on what else is in the batch, so its rows of the engine's logits must agree with
  the oracle's.

Tolerance: the stated one for bf16 models, 2e-2 of the row's largest |logit|. The weights and the KV cache are bf16;
the activation operands between the GEMMs are carried in half precision (with bf16 operands there the rounding
errors of 32 layers add up to 3.3e-2, measured), so what remains are the bf16 roundings inside the attention
(queries, cached keys and values, probabilities). The probes are sampled requests (temperature, top-k, top-p, Philox
seed as in the benchmark): every token is checked against the oracle's sampler run on the engine's own logits row of
128256 entries (exact, up to the fp32 arithmetic of the cumulative sums), and against the oracle's sampler on the oracle's
logits wherever no decision lies within twice the measured logit error of flipping (with candidates as dense as they are
in a vocabulary of this size, few tokens pass that second filter; the count is printed)."""
import numpy as np
import pytest

import synth
from oracle import model as M, sampling as S
from oracle.philox import uniform_for_token
from oracle.scheduler import Scheduler
from tests import parity

pytestmark = pytest.mark.gpu

N_PROBES, PROBE_LEN, NEW_TOKENS, N_DRAWN = 2, 16, 5, 80


def test_llama3_8b_shape_schedule_exact_and_probe_logits(lib):
    cfg, eng = synth.model_config("llama3_8b"), synth.engine_config("llama3_8b")
    raw = synth.make_weights(cfg, 1002)
    blob = synth.pack_blob(cfg, raw)
    drawn = synth.make_workload("llama3_8b", cfg["vocab"], 2002, n_requests=N_DRAWN)
    rng = np.random.default_rng(77)
    probes = [dict(drawn[i], prompt=rng.integers(0, cfg["vocab"], PROBE_LEN).astype(np.int32)) for i in range(N_PROBES)]
    reqs = probes + drawn
    for r in reqs:
        r["max_new_tokens"] = NEW_TOKENS
        r["arrival_s"] = 0.0
    assert max(len(r["prompt"]) for r in reqs) > 2048 and sum(len(r["prompt"]) for r in reqs) > 3 * eng["max_prefill_tokens"]

    sched = Scheduler.from_engine(eng)
    for r in reqs:
        sched.submit(r["prompt"], r["max_new_tokens"])
    # the probes alone, for the oracle's model: two requests, a pool that just holds them
    small = Scheduler(2 * N_PROBES, eng["kv_block_size"], N_PROBES, eng["max_prefill_tokens"], 8, -1)
    for r in probes:
        small.submit(r["prompt"], r["max_new_tokens"])
    W = M.Weights(cfg, raw)
    kv = M.PagedKV(cfg, 2 * N_PROBES, eng["kv_block_size"])

    D = lib.DBG
    e = lib.Engine(cfg, eng, blob, flags=lib.FLAG_TRACE | lib.FLAG_EXIT_WHEN_IDLE | lib.FLAG_KEEP_LOGITS)
    worst, kinds, probe_steps, biggest = 0.0, [], 0, 0
    sampled_checked = sampled_undecided = sampled_exact = 0
    try:
        for r in reqs:
            e.submit_request(r)
        for it in range(200):
            e.run(1)
            e.wait()
            plan = sched.step(len(reqs))
            sched.check_invariants()
            if plan.kind == 0:
                assert e.stats()["iterations"] == it
                break
            kinds.append((plan.kind, len(plan.tickets), len(plan.input_ids)))
            biggest = max(biggest, len(plan.input_ids))
            assert list(e.debug_read(D.INPUT_IDS, np.int32)) == plan.input_ids
            assert list(e.debug_read(D.POSITIONS, np.int32)) == plan.positions
            assert list(e.debug_read(D.SLOT_MAPPING, np.int32)) == plan.slot_mapping
            assert list(e.debug_read(D.SEQ_BATCH_SLOT, np.uint32)) == plan.batch_slots
            assert list(e.debug_read(D.SEQ_LENS, np.uint32)) == plan.seq_lens
            assert list(e.debug_read(D.CU_SEQLENS, np.uint32)) == plan.cu_seqlens
            fs = e.debug_read(D.FREE_STACK, np.uint32)
            assert fs[0] == len(sched.free) and list(fs[1:]) == sched.free
            bt = e.debug_read(D.BLOCK_TABLES, np.uint32).reshape(eng["max_batch"], -1)
            for b, blocks in zip(plan.batch_slots, plan.block_tables):
                assert list(bt[b][: len(blocks)]) == blocks
            evs = e.drain()
            by_ticket = {int(x["request_id"]): int(x["token"]) for x in evs}
            assert sorted(by_ticket) == sorted(plan.tickets)
            in_batch = [t for t in range(N_PROBES) if t in plan.tickets]
            if in_batch:
                assert in_batch == list(range(N_PROBES))        # admitted together, same length: they move in step
                sp = small.step(N_PROBES)
                assert sp.kind == plan.kind and sp.tickets == in_batch
                ref = M.paged_forward(cfg, W, kv, sp.input_ids, sp.positions, sp.slot_mapping, sp.tok_seq, sp.block_tables,
                                      sp.last_idx)
                got = e.debug_read(D.LOGITS, np.float32).reshape(len(plan.tickets), cfg["vocab"])
                rows = got[[plan.tickets.index(t) for t in in_batch]]
                err = np.abs(rows - ref).max(axis=1) / np.abs(ref).max(axis=1)
                worst = max(worst, float(err.max()))
                assert err.max() < 2e-2, (it, plan.kind, len(plan.input_ids), err)
                for j, t in enumerate(in_batch):
                    # the sampled token at V = 128256: exactly, against the oracle's sampler run on the engine's own logits
                    # (sampler parity given the same logits) ...
                    r = reqs[t]
                    assert r["temperature"] > 0
                    sampled_exact += int(parity.token_matches_own_logits(rows[j], r, sp.gen_index[j], by_ticket[t]))
                    # ... and against the oracle's sampler on the oracle's logits wherever an error of twice the one just
                    # measured for this row cannot move a decision
                    d = S.sample_detail(ref[j], r["temperature"], r["top_k"], r["top_p"], uniform_for_token(r["seed"], sp.gen_index[j]))
                    tol = 2.0 * float(np.abs(rows[j] - ref[j]).max())
                    if parity.sampling_decisions_clear(ref[j], r, d, tol):
                        assert by_ticket[t] == d["token"], (it, t, by_ticket[t], d["token"])
                        sampled_checked += 1
                    else:
                        sampled_undecided += 1
                small.commit(sp, [by_ticket[t] for t in in_batch])
                probe_steps += 1
            sched.commit(plan, [by_ticket[t] for t in plan.tickets])
        else:
            raise AssertionError("did not finish")
    finally:
        e.shutdown()
    assert probe_steps == NEW_TOKENS
    assert kinds[0][0] == 1 and kinds[0][2] > 2048 and biggest > eng["max_prefill_tokens"] // 2   # the probes' prefill shared a large iteration
    assert any(k == 2 and n > 64 for k, n, _ in kinds)                      # decode iterations beyond 64 sequences
    print("full size: iterations", kinds, "worst relative logit error of the probes", worst,
          "sampled probe tokens: equal to the oracle's sampler on the engine's logits", sampled_exact, "of", N_PROBES * NEW_TOKENS,
          "; on the oracle's logits: equal", sampled_checked, "undecided", sampled_undecided)
    assert sampled_exact >= N_PROBES * NEW_TOKENS - 2


def test_full_head_configuration_whole_context_items(lib):
    """The llama3_8b head configuration (32 q / 8 kv heads of 128) in one narrow layer, 172 sequences with contexts of 8 to
    2100 tokens: enough (sequence, kv head) pairs that the scheduler hands whole contexts to the decode attention by
    itself, longest first, about 1400 items on 256 workgroups, the long ones walked in up to five rounds. Every logits row
    of every iteration against the oracle, the work list against the plan."""
    cfg, eng = synth.model_config("mini_heads32"), synth.engine_config("mini_heads32")
    raw = synth.make_weights(cfg, 51, gain_jitter=0.1)
    blob = synth.pack_blob(cfg, raw)
    rng = np.random.default_rng(51)
    plens = [int(x) for x in rng.integers(8, 120, 172)]
    plens[:6] = [2100, 1100, 1030, 700, 511, 513]
    reqs = [dict(arrival_s=0.0, prompt=rng.integers(0, cfg["vocab"], P).astype(np.int32), max_new_tokens=3, temperature=0.0, top_k=0,
                 top_p=1.0, seed=i) for i, P in enumerate(plens)]
    modes = []
    worst = parity.stepwise_check(lib, cfg, eng, raw, blob, reqs, rtol=2e-2, item_modes=modes)
    print("full head configuration, whole contexts: worst relative logit error", worst, "item modes", modes)
    assert True in modes        # the decode iterations of the full batch took whole contexts


def test_free_running_loop_switches_between_the_two_chains(lib):
    """The llama3_8b head configuration in one narrow layer, 172 sequences served by the free-running loop (one window,
    HIP graphs, eight iterations enqueued ahead): while 128 or more sequences run the launcher takes the kernel chain
    without the merge kernels, before and after it the full chain, from a host view that is iterations old. The
    schedule is bit-exact and every token is the oracle's, teacher-forced, whichever chain an iteration ran on."""
    cfg, eng = synth.model_config("mini_heads32"), synth.engine_config("mini_heads32")
    raw = synth.make_weights(cfg, 52, gain_jitter=0.1)
    blob = synth.pack_blob(cfg, raw)
    rng = np.random.default_rng(52)
    plens = [int(x) for x in rng.integers(8, 120, 172)]
    plens[:4] = [1100, 700, 511, 513]
    reqs = [dict(arrival_s=0.0, prompt=rng.integers(0, cfg["vocab"], P).astype(np.int32), max_new_tokens=int(rng.integers(14, 40)),
                 temperature=0.0, top_k=0, top_p=1.0, seed=i) for i, P in enumerate(plens)]
    ev, trace, st = parity.run_engine(lib, cfg, eng, blob, reqs, poll_cap=1 << 16)
    assert st["n_running"] == 0 and st["free_blocks"] == eng["kv_num_blocks"]
    assert len(ev) == sum(r["max_new_tokens"] for r in reqs)
    res = parity.check_against_oracle(cfg, M.Weights(cfg, raw), eng, reqs, ev, trace, rtol=2e-2, tok_rtol=2e-3)
    dec = trace[trace["kind"] == 2]
    print("free run over both chains: tokens", res["tokens"], "near ties", res["near_ties"], "decode iterations with >= 128 sequences",
          int((dec["n_seqs"] >= 128).sum()), "with fewer", int((dec["n_seqs"] < 128).sum()))
    assert (dec["n_seqs"] >= 128).sum() >= 12 and (dec["n_seqs"] < 128).sum() >= 12    # longer than the launcher's lead of eight iterations
    assert res["near_ties"] <= res["tokens"] // 8      # token tolerance 2e-3 of the largest logit, as in the other end-to-end tests
