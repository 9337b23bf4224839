"""Parity at the full width of the mixture-of-experts benchmark model: one layer of the moe_30b_a3b shape (d 2048, 32 q /
4 kv heads of 128, 128 experts of width 768, 8 active, vocabulary 151 936; 48 such layers make the benchmark's model),
so the grouped GEMMs run their real shapes (1536 x 2048 and 2048 x 768 per expert, 128 groups).

One prefill iteration of about 1000 tokens gives the experts 62 tokens on average: about half of them run as independent
wave items (three or four token blocks), the others as tile GEMMs. One decode iteration of 42 sequences follows (two or
three tokens per expert). The oracle cannot afford the expert loop for a thousand tokens, and with one layer it need
not: keys and values of the layer depend on the embeddings only, so the residual stream after the layer is computed for a
SAMPLE of the tokens (attention over the whole context, experts for those tokens only, fed with the engine's routing)
and compared with the engine's (BLINK_DBG_HIDDEN); the logits are compared for every sequence. The scheduler's metadata
is checked in full."""
import numpy as np
import pytest

import synth
from oracle import model as M
from oracle.scheduler import Scheduler
from tests import parity

pytestmark = pytest.mark.gpu


def test_moe_30b_a3b_width_sampled_tokens(lib):
    cfg = dict(synth.model_config("moe_30b_a3b"), n_layers=1)
    eng = dict(kv_block_size=16, kv_num_blocks=160, max_batch=48, max_seq_len=400, max_prefill_tokens=1100, ring_slots=64, eos_token_id=-1)
    raw = synth.make_weights(cfg, 1004, gain_jitter=0.1, threads=16)
    blob = synth.pack_blob(cfg, raw)
    rng = np.random.default_rng(9)
    lens = [330, 290] + [int(x) for x in rng.integers(3, 17, 40)]
    reqs = [dict(arrival_s=0.0, prompt=rng.integers(0, cfg["vocab"], P).astype(np.int32), max_new_tokens=2, temperature=0.0, top_k=0,
                 top_p=1.0, seed=i) for i, P in enumerate(lens)]
    W = M.Weights(cfg, raw)
    sched = Scheduler.from_engine(eng)
    for r in reqs:
        sched.submit(r["prompt"], r["max_new_tokens"])
    D = lib.DBG
    stats = dict(pairs=0, unclear=0)
    hist = {}                                   # ticket -> token ids of its context so far
    e = lib.Engine(cfg, eng, blob, flags=lib.FLAG_TRACE | lib.FLAG_EXIT_WHEN_IDLE | lib.FLAG_KEEP_LOGITS)
    try:
        for r in reqs:
            e.submit_request(r)
        for it in range(2):
            e.run(1)
            e.wait()
            plan = sched.step(len(reqs))
            sched.check_invariants()
            assert plan.kind == (1 if it == 0 else 2) and len(plan.tickets) == len(reqs)
            assert list(e.debug_read(D.INPUT_IDS, np.int32)) == plan.input_ids
            assert list(e.debug_read(D.POSITIONS, np.int32)) == plan.positions
            assert list(e.debug_read(D.SLOT_MAPPING, np.int32)) == plan.slot_mapping
            assert list(e.debug_read(D.CU_SEQLENS, np.uint32)) == plan.cu_seqlens
            T = len(plan.input_ids)
            routing = e.debug_read(D.ROUTING, np.uint32).reshape(1, T, cfg["n_active"])
            hidden = e.debug_read(D.HIDDEN, np.float32).reshape(T, cfg["d_model"])
            logits = e.debug_read(D.LOGITS, np.float32).reshape(len(plan.sample_seq), cfg["vocab"])
            counts = np.bincount(routing.reshape(-1), minlength=cfg["n_experts"])
            if it == 0:
                assert (counts > 64).sum() >= 20 and ((counts > 0) & (counts <= 64)).sum() >= 20, counts   # both kinds of experts
            for si, t in enumerate(plan.tickets):
                hist.setdefault(t, []).extend(plan.input_ids[plan.cu_seqlens[si]:plan.cu_seqlens[si + 1]])
            # sample: the last token of every sequence and 40 other tokens of the iteration
            sample = sorted(set(plan.last_idx) | set(int(x) for x in rng.integers(0, T, 40)))
            x_ref = np.empty((len(sample), cfg["d_model"]))
            x_in = np.empty((len(sample), cfg["d_model"]))
            attn = np.empty((len(sample), cfg["n_q_heads"], cfg["head_dim"]))
            kv_of = {}
            for i, tk in enumerate(sample):
                si = plan.tok_seq[tk]
                t = plan.tickets[si]
                if t not in kv_of:              # keys and values of the sequence's whole context, from the embeddings
                    ids = np.asarray(hist[t])
                    _, k, v = M._qkv(cfg, W, 0, W["embed"][ids], np.arange(ids.size))
                    kv_of[t] = (k, v)
                p = plan.positions[tk]
                x0 = W["embed"][np.asarray([plan.input_ids[tk]])]
                q, _, _ = M._qkv(cfg, W, 0, x0, np.asarray([p]))
                attn[i] = M._attend(cfg, q[0], kv_of[t][0][: p + 1], kv_of[t][1][: p + 1])
                x_in[i] = x0[0]
            log = []
            x_ref = M._post_attention(cfg, W, 0, x_in, attn, routing=[routing[0][sample]], route_log=log)
            parity.check_routing(cfg, routing[:, sample], log, stats)
            err_h = np.abs(hidden[sample] - x_ref).max(axis=1) / np.abs(x_ref).max(axis=1)
            rows = [sample.index(li) for li in plan.last_idx]
            ref_logits = M._head(cfg, W, x_ref[rows])
            err_l = np.abs(logits - ref_logits).max(axis=1) / np.abs(ref_logits).max(axis=1)
            print("iteration", it, "tokens", T, "experts with > 64 tokens", int((counts > 64).sum()), "sampled tokens", len(sample),
                  "worst hidden error", float(err_h.max()), "worst logit error", float(err_l.max()))
            assert err_h.max() < 2e-2 and err_l.max() < 2e-2
            evs = e.drain()
            by_ticket = {int(x["request_id"]): int(x["token"]) for x in evs}
            for i, t in enumerate(plan.sample_tickets):
                parity.token_matches_own_logits(logits[i], reqs[t], plan.gen_index[i], by_ticket[t])
            sched.commit(plan, [by_ticket[t] for t in plan.sample_tickets])
        assert stats["unclear"] <= 0.08 * stats["pairs"], stats
    finally:
        e.shutdown()
