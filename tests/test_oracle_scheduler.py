"""Pins for the oracle's scheduler: a schedule worked out by hand, invariants under random load,
emission counts, FCFS head-of-line blocking, window restarts, and service == per-request generation."""
import numpy as np
import pytest

import synth
from oracle import model as M, serve as SV
from oracle.scheduler import Scheduler, PREFILL, DECODE, IDLE, blocks_needed, LEGAL_EDGES


def req(P, n, first=0):
    return dict(prompt=np.arange(first, first + P) % 50, max_new_tokens=n, temperature=0.0, top_k=0, top_p=1.0, seed=0)


def test_reservation_formula():
    assert blocks_needed(20, 3, 16) == 2 and blocks_needed(10, 8, 16) == 2 and blocks_needed(5, 2, 16) == 1
    assert blocks_needed(16, 1, 16) == 1 and blocks_needed(16, 2, 16) == 2 and blocks_needed(1, 1, 16) == 1


def test_hand_worked_three_requests_pool_of_four():
    """bs 16, 4 blocks, 2 batch slots; requests (P, max_new) = (20,3), (10,8), (5,2).
    Worked by hand from the iteration rules: see the expected table below."""
    s = Scheduler(4, 16, 2, 8192, 8)
    plans = []
    SV.run_schedule(s, [req(20, 3), req(10, 8), req(5, 2)], lambda pl: [7] * len(pl.tickets), on_plan=plans.append)
    # iteration: (kind, tickets, batch slots, positions of each sequence's last token, block tables, free after)
    exp = [
        (PREFILL, [0, 1], [0, 1], [19, 9], [[0, 1], [2]], 1),
        (DECODE, [0, 1], [0, 1], [20, 10], [[0, 1], [2]], 1),
        (DECODE, [0, 1], [0, 1], [21, 11], [[0, 1], [2]], 1),      # request 0 emits its 3rd token
        (PREFILL, [2], [0], [4], [[1]], 2),                        # blocks 0,1 pushed back; pop returns 1
        (DECODE, [2, 1], [0, 1], [5, 12], [[1], [2]], 2),          # request 2 done
        (DECODE, [1], [1], [13], [[2]], 3),
        (DECODE, [1], [1], [14], [[2]], 3),
        (DECODE, [1], [1], [15], [[2]], 3),
        (DECODE, [1], [1], [16], [[2, 1]], 2),                     # crosses a block boundary: pop returns 1
    ]
    assert len(plans) == len(exp)
    for pl, e in zip(plans, exp):
        got = (pl.kind, pl.tickets, pl.batch_slots, [pl.positions[i] for i in pl.last_idx], pl.block_tables, pl.free_blocks_after)
        assert got == e, (pl.iteration, got, e)
    assert plans[0].slot_mapping[:20] == list(range(0, 20)) and plans[0].slot_mapping[20:] == list(range(32, 42))
    assert plans[0].cu_seqlens == [0, 20, 30] and plans[0].tok_seq == [0] * 20 + [1] * 10
    assert plans[8].slot_mapping == [16] and plans[8].input_ids == [7]
    assert plans[3].admitted == [2] and plans[0].admitted == [0, 1]
    assert [len(s.outputs[t]) for t in range(3)] == [3, 8, 2]
    s.step(3)
    assert s.free == [3, 0, 2, 1] and s.committed == 0


def test_head_of_line_blocks_and_prefill_budget():
    # ticket 1 needs more blocks than are uncommitted: ticket 2, which would fit, must wait behind it
    s = Scheduler(6, 16, 4, 8192, 8)
    plans = []
    SV.run_schedule(s, [req(40, 9), req(60, 10), req(3, 2)], lambda pl: [1] * len(pl.tickets), on_plan=plans.append)
    assert plans[0].admitted == [0]
    first_adm_1 = next(p.iteration for p in plans if 1 in p.admitted)
    first_adm_2 = next(p.iteration for p in plans if 2 in p.admitted)
    assert first_adm_1 == 9 and first_adm_2 == 9      # after request 0 retires, both fit
    # prefill token budget: the first request is exempt, the next must fit in the remainder
    s = Scheduler(64, 16, 4, 50, 8)
    plans = []
    SV.run_schedule(s, [req(70, 2), req(10, 2), req(30, 2), req(30, 2)], lambda pl: [1] * len(pl.tickets), on_plan=plans.append)
    assert plans[0].admitted == [0] and plans[1].admitted == [1, 2] and plans[2].admitted == [3]


def test_eos_is_emitted_and_counted():
    s = Scheduler(8, 16, 2, 8192, 8, eos_token_id=9)
    seq = iter([1, 2, 9, 4, 5])
    ev = SV.run_schedule(s, [req(4, 10)], lambda pl: [next(seq)])
    assert s.outputs[0] == [1, 2, 9] and ev[-1][-1] is True


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_invariants_random_load_and_exact_counts(seed):
    rng = np.random.default_rng(seed)
    n = 60
    reqs = [req(int(rng.integers(1, 70)), int(rng.integers(1, 20))) for _ in range(n)]
    need_max = max(blocks_needed(len(r["prompt"]), r["max_new_tokens"], 16) for r in reqs)
    s = Scheduler(max(need_max, 12), 16, 5, 100, 16, eos_token_id=3)
    tok_rng = np.random.default_rng(seed + 100)
    peak = [0]

    def on_plan(pl):
        assert s.n_running() <= 5
        peak[0] = max(peak[0], s.committed)
        assert pl.admitted == sorted(pl.admitted)
        assert pl.kind in (PREFILL, DECODE)
        if pl.kind == PREFILL:
            assert sorted(pl.tickets) == sorted(pl.admitted)
        # slot mapping addresses each sequence's own blocks only
        for t, sl in enumerate(pl.slot_mapping):
            assert sl // 16 in pl.block_tables[pl.tok_seq[t]]
        assert len(set(pl.slot_mapping)) == len(pl.slot_mapping)

    ev = SV.run_schedule(s, reqs, lambda pl: list(tok_rng.integers(0, 12, len(pl.tickets))), on_plan=on_plan)
    admitted_order = [t for (t, a, b) in s.transitions if b == 2]
    assert admitted_order == list(range(n))
    for t in range(n):
        out = s.outputs[t]
        exp = reqs[t]["max_new_tokens"]
        if 3 in out:
            exp = min(exp, out.index(3) + 1)
        assert len(out) == exp
    assert all((a, b) in LEGAL_EDGES for _, a, b in s.transitions)
    assert peak[0] <= s.n_blocks
    # events: per request consecutive indices, exactly one first and one last
    for t in range(n):
        mine = [e for e in ev if e[1] == t]
        assert [e[2] for e in mine] == list(range(len(mine)))
        assert [e[4] for e in mine].count(True) == 1 and mine[-1][5] is True


def test_windowed_run_equals_single_run():
    """State survives stopping the loop every few iterations (section 4.2, window recovery)."""
    rng = np.random.default_rng(5)
    reqs = [req(int(rng.integers(1, 40)), int(rng.integers(1, 12))) for _ in range(20)]
    f = lambda pl: [(pl.iteration * 7 + b) % 11 for b in pl.batch_slots]
    s1 = Scheduler(16, 16, 4, 64, 8)
    e1 = SV.run_schedule(s1, reqs, f)
    s2 = Scheduler(16, 16, 4, 64, 8)
    for r in reqs:
        s2.submit(r["prompt"], r["max_new_tokens"])
    e2 = []
    while True:
        for _ in range(3):                       # a window of 3 iterations
            pl = s2.step(len(reqs))
            if pl.kind == IDLE:
                break
            e2 += [(pl.iteration,) + e for e in s2.commit(pl, f(pl))]
        if pl.kind == IDLE:
            break
    assert e1 == e2


def test_service_equals_per_request_generation_and_replay_tails():
    cfg = dict(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=50, dtype=0,
               rms_eps=1e-5, rope_theta=10000.0)
    W = M.Weights(cfg, synth.make_weights(cfg, 11, std=0.3))
    rng = np.random.default_rng(6)
    reqs = []
    for i in range(7):
        r = req(int(rng.integers(1, 30)), int(rng.integers(1, 9)), first=i * 3)
        if i % 2:
            r.update(temperature=0.8, top_k=5, top_p=0.9, seed=synth.splitmix64(3, i))
        reqs.append(r)
    eng = dict(kv_block_size=4, kv_num_blocks=24, max_batch=3, max_prefill_tokens=40, ring_slots=8, eos_token_id=-1)
    ev, s = SV.serve(cfg, W, eng, reqs)
    for t, r in enumerate(reqs):
        assert s.outputs[t] == SV.generate_reference(cfg, W, r)
    # arrivals trickling in (tails per iteration) change the schedule but not the streams
    tails = [1, 1, 2, 2, 4, 4, 4, 7]
    ev2, s2 = SV.serve(cfg, W, eng, reqs, tails=tails)
    assert [s2.outputs[t] for t in range(7)] == [s.outputs[t] for t in range(7)]
    assert [e[0] for e in ev2] != [e[0] for e in ev]


def test_churn_pool_constant_is_what_the_oracle_side_script_computes():
    """The Churn engine's pool (60 % of the peak demand of its request set) is a stored number: it must be the one
    oracle.churn_pool derives from the oracle's reservation rule, and at least the largest single reservation."""
    import synth
    from oracle.churn_pool import churn_pool_blocks
    cfg, eng = synth.model_config("churn"), synth.engine_config("churn")
    reqs = synth.make_workload("churn", cfg["vocab"], 2001)
    assert churn_pool_blocks(reqs, eng["kv_block_size"]) == eng["kv_num_blocks"]
    assert eng["kv_num_blocks"] >= max(blocks_needed(len(r["prompt"]), r["max_new_tokens"], 16) for r in reqs)


# ---- chunked prefill with mixed iterations ---------------------------------------------------------------------------

def test_chunked_hand_worked_three_requests_budget_24():
    """bs 16, 8 blocks, 3 batch slots, 24 tokens per iteration; requests (P, max_new) = (20,2), (30,2), (5,3), all there
    at the start. Worked by hand from the rules of the chunked mode:
      it 0: admit A (20 tokens, the whole prompt) and B (the 4 tokens the budget still holds); A samples.
      it 1: A decodes (1 token), B takes the other 23; nothing is admitted (budget spent); A's second token ends it.
      it 2: A retires (blocks 0,1 back; slot 0 free); B takes its last 3 tokens; C is admitted into slot 0 with its 5
            tokens; the sequences run in batch-slot order, so C (slot 0) comes before B (slot 1); both sample.
      it 3: B and C decode; B ends.   it 4: B retires; C decodes its third token and ends."""
    s = Scheduler(8, 16, 3, 24, 8, chunked=True)
    plans = []
    SV.run_schedule(s, [req(20, 2), req(30, 2), req(5, 3)], lambda pl: [7] * len(pl.sample_seq), on_plan=plans.append)
    # (kind, tickets, batch slots, first position per sequence, tokens per sequence, sampling tickets, block tables, free after)
    exp = [
        (PREFILL, [0, 1], [0, 1], [0, 0], [20, 4], [0], [[0, 1], [2]], 5),
        (PREFILL, [0, 1], [0, 1], [20, 4], [1, 23], [0], [[0, 1], [2, 3]], 4),
        (PREFILL, [2, 1], [0, 1], [0, 27], [5, 3], [2, 1], [[1], [2, 3]], 5),     # stack after the retire: .., 0, 1 -> pop gives 1
        (DECODE, [2, 1], [0, 1], [5, 30], [1, 1], [2, 1], [[1], [2, 3]], 5),
        (DECODE, [2], [0], [6], [1], [2], [[1]], 7),
    ]
    assert len(plans) == len(exp)
    for pl, e in zip(plans, exp):
        per_seq = [pl.cu_seqlens[i + 1] - pl.cu_seqlens[i] for i in range(len(pl.tickets))]
        got = (pl.kind, pl.tickets, pl.batch_slots, pl.pos0, per_seq, pl.sample_tickets, pl.block_tables, pl.free_blocks_after)
        assert got == e, (pl.iteration, got, e)
    assert plans[0].admitted == [0, 1] and plans[1].admitted == [] and plans[2].admitted == [2]
    assert plans[1].positions == [20] + list(range(4, 27)) and plans[1].slot_mapping == [20] + list(range(36, 48)) + list(range(48, 59))
    assert plans[1].input_ids == [7] + [int(x) for x in req(30, 2)["prompt"][4:27]]
    assert plans[2].positions == list(range(5)) + [27, 28, 29] and plans[2].last_idx == [4, 7] and plans[2].gen_index == [0, 0]
    assert plans[3].input_ids == [7, 7] and plans[3].gen_index == [1, 1]
    assert [len(s.outputs[t]) for t in range(3)] == [2, 2, 3]
    s.step(3)
    assert s.free == [7, 6, 5, 4, 0, 2, 3, 1] and s.committed == 0


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_chunked_invariants_under_random_load(seed):
    """Blocks are conserved, the budget holds, at most one request is part-way through its prompt at the start of an
    iteration, a decoding request gets a token in EVERY iteration until it ends (nothing pauses), prompts are processed
    in order without gaps, admissions are in ticket order, and every request emits exactly its count."""
    rng = np.random.default_rng(seed)
    n = 50
    reqs = [req(int(rng.integers(1, 90)), int(rng.integers(1, 12))) for _ in range(n)]
    need_max = max(blocks_needed(len(r["prompt"]), r["max_new_tokens"], 16) for r in reqs)
    budget = 40
    s = Scheduler(max(need_max, 14), 16, 5, budget, 16, chunked=True)
    done_prompt, last_decode_iter, admitted_order = {}, {}, []
    plans = []

    def on_plan(pl):
        plans.append(pl)
        assert 0 < len(pl.input_ids) <= budget
        part = [b for b in range(s.max_batch) if s.running[b] is not None and 0 < s.running[b].prefilled < s.running[b].P]
        assert len(part) <= 1
        admitted_order.extend(pl.admitted)
        for i, t in enumerate(pl.tickets):
            ntok = pl.cu_seqlens[i + 1] - pl.cu_seqlens[i]
            P = len(reqs[t]["prompt"])
            if done_prompt.get(t, 0) < P:                  # a prompt chunk: continues exactly where the last one ended
                assert pl.pos0[i] == done_prompt.get(t, 0) and ntok >= 1
                assert pl.input_ids[pl.cu_seqlens[i]:pl.cu_seqlens[i + 1]] == [int(x) for x in reqs[t]["prompt"][pl.pos0[i]:pl.pos0[i] + ntok]]
                done_prompt[t] = pl.pos0[i] + ntok
                assert (i in pl.sample_seq) == (done_prompt[t] == P)
                if done_prompt[t] == P:
                    last_decode_iter[t] = pl.iteration
            else:                                          # a decode: one token, in the iteration right after its last one
                assert ntok == 1 and i in pl.sample_seq and pl.iteration == last_decode_iter[t] + 1
                last_decode_iter[t] = pl.iteration

    SV.run_schedule(s, reqs, lambda pl: [int(rng.integers(0, 50)) for _ in pl.sample_seq], on_plan=on_plan)
    assert admitted_order == list(range(n))
    assert [len(s.outputs[t]) for t in range(n)] == [r["max_new_tokens"] for r in reqs]
    s.step(n)
    assert sorted(s.free) == list(range(s.n_blocks)) and s.committed == 0
    assert any(pl.kind == PREFILL and len(pl.sample_seq) > 1 and len(pl.tickets) > len(pl.admitted) for pl in plans)   # mixed iterations occurred


def test_chunked_equals_unchunked_when_everything_fits_one_iteration():
    """With a budget that holds all prompts at once the chunked schedule is the plain one, iteration by iteration
    (and the plain scheduler is pinned above)."""
    reqs = [req(20, 3), req(10, 5, first=7), req(33, 2, first=11)]
    a, b = Scheduler(16, 16, 4, 8192, 8), Scheduler(16, 16, 4, 8192, 8, chunked=True)
    pa, pb = [], []
    SV.run_schedule(a, reqs, lambda pl: [5] * len(pl.sample_seq), on_plan=pa.append)
    SV.run_schedule(b, reqs, lambda pl: [5] * len(pl.sample_seq), on_plan=pb.append)
    assert len(pa) == len(pb)
    for x, y in zip(pa, pb):
        for f in ("kind", "tickets", "batch_slots", "input_ids", "positions", "slot_mapping", "tok_seq", "cu_seqlens", "last_idx",
                  "block_tables", "gen_index", "sample_seq", "free_blocks_after", "admitted"):
            assert getattr(x, f) == getattr(y, f), (x.iteration, f)


def test_chunked_service_equals_per_request_generation():
    """The model side of chunking: a prompt fed through the paged forward pass in several chunks, mixed with other
    requests' decode tokens, gives the token streams of every request generated alone with a contiguous cache."""
    cfg = dict(synth.model_config("tiny"), n_layers=2, vocab=97, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96)
    raw = synth.make_weights(cfg, 5, gain_jitter=0.1)
    W = M.Weights(cfg, raw)
    rng = np.random.default_rng(3)
    reqs = [dict(prompt=rng.integers(0, 97, P).astype(np.int32), max_new_tokens=n, temperature=0.0, top_k=0, top_p=1.0, seed=0)
            for P, n in ((37, 4), (5, 6), (50, 3), (18, 5))]
    eng = dict(kv_block_size=16, kv_num_blocks=24, max_batch=3, max_prefill_tokens=20, ring_slots=8, eos_token_id=-1, chunked_prefill=True)
    ev, sched = SV.serve(cfg, W, eng, reqs)
    assert max(len(p) for p in [r["prompt"] for r in reqs]) > 2 * eng["max_prefill_tokens"]     # prompts span three iterations
    for t, r in enumerate(reqs):
        assert sched.outputs[t] == SV.generate_reference(cfg, W, r), t


# ---- on-demand KV growth with preemption --------------------------------------------------------------------------------

def test_preemption_hand_worked_three_requests_pool_of_four():
    """bs 16, 4 blocks, 3 batch slots; requests (P, max_new) = (16,20), (16,4), (10,3), all there at the start. By hand:
      it 0: all three fit (one block each, no worst-case reservation): blocks A [0], B [1], C [2]; one block left.
      it 1: A and B have filled their block and need one more each, one is free: the highest ticket, C, is preempted
            (its block 2 goes back on top of the stack); A takes 2, B takes 3.
      it 2, 3: C needs one block to come back and none is free: it waits (and no one else could be admitted either);
            A and B decode; B emits its fourth token in it 3.
      it 4: B retires (1, 3 back), C resumes into slot 1 by recomputing its 10 prompt tokens + its one output token, block 3;
            it samples output index 1; A is paused for this prefill iteration.
      it 5: A and C decode; C ends. Then A decodes alone, takes block 3 when its context reaches 32, and ends."""
    s = Scheduler(4, 16, 3, 8192, 8, preempt=True)
    plans = []
    SV.run_schedule(s, [req(16, 20), req(16, 4), req(10, 3)], lambda pl: [7] * len(pl.sample_seq), on_plan=plans.append)
    exp = [   # kind, tickets, batch slots, admitted, resumed, preempted, block tables, free after, gen index
        (PREFILL, [0, 1, 2], [0, 1, 2], [0, 1, 2], [], [], [[0], [1], [2]], 1, [0, 0, 0]),
        (DECODE, [0, 1], [0, 1], [], [], [2], [[0, 2], [1, 3]], 0, [1, 1]),
        (DECODE, [0, 1], [0, 1], [], [], [], [[0, 2], [1, 3]], 0, [2, 2]),
        (DECODE, [0, 1], [0, 1], [], [], [], [[0, 2], [1, 3]], 0, [3, 3]),
        (PREFILL, [2], [1], [], [2], [], [[3]], 1, [1]),
        (DECODE, [0, 2], [0, 1], [], [], [], [[0, 2], [3]], 1, [4, 2]),
    ]
    for pl, e in zip(plans, exp):
        got = (pl.kind, pl.tickets, pl.batch_slots, pl.admitted, pl.resumed, pl.preempted, pl.block_tables, pl.free_blocks_after, pl.gen_index)
        assert got == e, (pl.iteration, got, e)
    assert plans[4].input_ids == [int(x) for x in req(10, 3)["prompt"]] + [7] and plans[4].positions == list(range(11))
    assert plans[4].slot_mapping == list(range(48, 59)) and plans[4].last_idx == [10]
    assert [len(s.outputs[t]) for t in range(3)] == [20, 4, 3]
    grow = next(pl for pl in plans if pl.tickets == [0] and len(pl.block_tables[0]) == 3)
    assert grow.positions == [32] and grow.block_tables == [[0, 2, 3]]
    s.step(3)
    assert sorted(s.free) == [0, 1, 2, 3] and not s.preempted


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_preemption_invariants_under_random_load(seed):
    """A pool far below the worst-case demand: blocks are conserved, every request emits exactly its count with output
    indices 0,1,2,.. in order (a stream continues where it stopped), a resumed request prefills its prompt followed by
    its own outputs, only the highest tickets are preempted, resumptions come before admissions, and preemptions occur."""
    rng = np.random.default_rng(seed)
    n = 40
    reqs = [req(int(rng.integers(1, 60)), int(rng.integers(4, 40))) for _ in range(n)]
    need_max = max(blocks_needed(len(r["prompt"]), r["max_new_tokens"], 16) for r in reqs)
    s = Scheduler(need_max + 3, 16, 6, 200, 16, preempt=True)
    next_index = {t: 0 for t in range(n)}
    stats = dict(preempted=0, resumed=0)

    def on_plan(pl):
        stats["preempted"] += len(pl.preempted)
        stats["resumed"] += len(pl.resumed)
        running_tickets = [r.ticket for r in s.running if r is not None]
        for v in pl.preempted:
            assert all(v > t for t in running_tickets)          # the victims were the most recently submitted
        if pl.admitted:
            assert not s.preempted                               # nobody waits preempted while a new ticket is admitted
        for i, t in zip(pl.sample_seq, pl.sample_tickets):
            assert pl.gen_index[pl.sample_seq.index(i)] == next_index[t]
            next_index[t] += 1
        for i, t in enumerate(pl.tickets):
            if t in pl.resumed:
                toks = pl.input_ids[pl.cu_seqlens[i]:pl.cu_seqlens[i + 1]]
                assert toks == [int(x) for x in reqs[t]["prompt"]] + s.outputs[t]

    SV.run_schedule(s, reqs, lambda pl: [int(rng.integers(0, 50)) for _ in pl.sample_seq], on_plan=on_plan)
    assert [len(s.outputs[t]) for t in range(n)] == [r["max_new_tokens"] for r in reqs]
    assert stats["preempted"] > 0 and stats["preempted"] == stats["resumed"]
    s.step(n)
    assert sorted(s.free) == list(range(s.n_blocks)) and not s.preempted


def test_preemption_mode_equals_plain_mode_when_the_pool_never_binds():
    reqs = [req(20, 3), req(10, 5, first=7), req(33, 2, first=11), req(5, 9, first=3)]
    a, b = Scheduler(64, 16, 3, 8192, 8), Scheduler(64, 16, 3, 8192, 8, preempt=True)
    pa, pb = [], []
    SV.run_schedule(a, reqs, lambda pl: [5] * len(pl.sample_seq), on_plan=pa.append)
    SV.run_schedule(b, reqs, lambda pl: [5] * len(pl.sample_seq), on_plan=pb.append)
    assert len(pa) == len(pb)
    for x, y in zip(pa, pb):
        for f in ("kind", "tickets", "batch_slots", "input_ids", "positions", "slot_mapping", "tok_seq", "cu_seqlens", "last_idx",
                  "block_tables", "gen_index", "sample_seq", "free_blocks_after", "admitted"):
            assert getattr(x, f) == getattr(y, f), (x.iteration, f)
        assert not y.preempted and not y.resumed


def test_preempted_service_equals_per_request_generation():
    """The model side of recomputation: a request that is preempted and later resumed by prefilling prompt + outputs so
    far continues with exactly the tokens it would have generated alone."""
    cfg = dict(synth.model_config("tiny"), n_layers=2, vocab=97, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96)
    raw = synth.make_weights(cfg, 6, gain_jitter=0.1)
    W = M.Weights(cfg, raw)
    rng = np.random.default_rng(4)
    reqs = [dict(prompt=rng.integers(0, 97, P).astype(np.int32), max_new_tokens=n, temperature=0.0, top_k=0, top_p=1.0, seed=0)
            for P, n in ((16, 30), (16, 12), (10, 20), (30, 8))]
    eng = dict(kv_block_size=16, kv_num_blocks=5, max_batch=3, max_prefill_tokens=100, ring_slots=8, eos_token_id=-1, preemption=True)
    seen = []
    ev, sched = SV.serve(cfg, W, eng, reqs, on_plan=lambda pl: seen.extend(pl.preempted))
    assert seen                                                   # somebody was preempted
    for t, r in enumerate(reqs):
        assert sched.outputs[t] == SV.generate_reference(cfg, W, r), t


# ---- prefix caching --------------------------------------------------------------------------------------------------

def test_prefix_hash_is_splitmix64_finalizer_and_chain():
    """mix64 is the output function of splitmix64: with the generator's increment as input it gives the generator's
    published first outputs for seed 0. The block hash is a polynomial in (token + 1) with the same increment as
    multiplier, mixed once; the chain mixes the previous key xor the block hash."""
    from oracle.scheduler import mix64, prefix_block_hash, prefix_chain, PREFIX_H0
    g = 0x9E3779B97F4A7C15
    assert mix64(g) == 0xE220A8397B1DCDAF and mix64(2 * g) == 0x6E789E6AA1B965F4 and mix64(3 * g) == 0x06C45D188009454F
    assert prefix_block_hash([]) == mix64(0) == 0
    assert prefix_block_hash([5]) == mix64(6)
    assert prefix_block_hash([5, 9]) == mix64((6 * g + 10) % 2 ** 64)
    assert prefix_chain(PREFIX_H0, [5, 9]) == mix64(PREFIX_H0 ^ prefix_block_hash([5, 9]))
    assert prefix_block_hash([0, 1]) != prefix_block_hash([1, 0]) != prefix_block_hash([0, 1, 0])


def _drive(s, n_visible, token=7):
    plan = s.step(n_visible)
    s.check_invariants()
    if plan.kind != IDLE:
        s.commit(plan, [token] * len(plan.sample_seq))
    return plan


def test_prefix_cache_hand_worked_sharing_idle_reuse_and_eviction():
    """bs 4, 8 blocks, 2 batch slots. Worked by hand from the rules in the scheduler's header."""
    s = Scheduler(8, 4, 2, 8192, 8, prefix_cache=True)
    A = list(range(1, 11))                                  # 10 tokens, two full blocks
    B = list(range(1, 9)) + [20, 21, 22]                    # shares A's two full blocks, but arrives in the same iteration
    C = [1, 2, 3, 4, 30, 31, 32, 33, 34]                    # shares A's first block
    for p, n in ((A, 2), (B, 1), (C, 2)):
        s.submit(p, n)
    p0 = _drive(s, 3)
    assert (p0.kind, p0.tickets, p0.block_tables, p0.free_blocks_after) == (PREFILL, [0, 1], [[0, 1, 2], [3, 4, 5]], 2)
    assert sorted(s.table.values()) == [0, 1] and s.pinned == 2 and s.committed == 1 + 3      # B's copies stay private
    p1 = _drive(s, 3)                                       # B retired (3, 4, 5 back on top); C matches block 0
    assert (p1.kind, p1.tickets, p1.batch_slots, p1.block_tables) == (PREFILL, [2], [1], [[0, 5, 4]])
    assert p1.positions == [4, 5, 6, 7, 8] and p1.slot_mapping == [20, 21, 22, 23, 16] and p1.pos0 == [4] and p1.input_ids == C[4:]
    assert p1.last_idx == [4] and p1.seq_lens == [9] and s.ref[0] == 2 and s.free == [7, 6, 3]
    assert sorted(s.table.values()) == [0, 1, 5] and s.pinned == 3 and s.committed == 1 + 1 and s.cache_hits == 1
    p2 = _drive(s, 3)
    assert (p2.kind, p2.tickets, p2.slot_mapping) == (DECODE, [0, 2], [10, 17])
    p3 = _drive(s, 3)                                       # both retire: private blocks on top, idle cached ones to the bottom
    assert p3.kind == IDLE and s.free == [0, 5, 1, 7, 6, 3, 2, 4] and s.pinned == 0 and s.committed == 0 and len(s.table) == 3
    D = list(range(1, 14))                                  # 13 tokens: matches A's two blocks, both idle
    s.submit(D, 1)
    p4 = _drive(s, 4)
    assert (p4.kind, p4.tickets, p4.block_tables, p4.positions) == (PREFILL, [3], [[0, 1, 3, 6]], [8, 9, 10, 11, 12])
    assert p4.slot_mapping == [12, 13, 14, 15, 24] and s.free == [4, 5, 2, 7] and s.pinned == 3 and s.committed == 1
    p5 = _drive(s, 4)
    assert p5.kind == IDLE and s.free == [0, 1, 3, 4, 5, 2, 7, 6] and len(s.table) == 4
    s.submit(list(range(40, 60)), 1)                        # 20 fresh tokens: five blocks, the fourth pop evicts C's block 5
    p6 = _drive(s, 5)
    assert p6.block_tables == [[6, 7, 2, 5, 4]] and s.evictions == 1 and sorted(s.table.values()) == [0, 1, 2, 3, 4, 5, 6, 7]
    assert s.free == [0, 1, 3]
    # (all five blocks of the new prompt are full and were entered: every block is cached now, three of them idle)
    s.submit(list(range(1, 6)), 1)                          # 5 tokens: matches block 0 (idle)
    p7 = _drive(s, 6)
    # the five blocks of the retired request went to the bottom in reverse table order: [6, 7, 2, 5, 4, 0, 1, 3]; the match
    # takes block 0 out (the top, 3, fills its place) and the one new block is the top, 1: A's second block is evicted
    assert p7.tickets == [5] and p7.block_tables == [[0, 1]] and s.evictions == 2 and s.free == [6, 7, 2, 5, 4, 3]


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_prefix_cache_invariants_and_no_shared_prefix_reduces_to_plain(seed):
    """Random load with shared prefixes behind a small pool: the invariants hold after every step, blocks are matched and
    evicted, every request gets all its tokens. The same load with distinct prompts (no repeated block anywhere) makes
    the same admissions, kinds and token counts as the plain scheduler: capacity accounting is unchanged when nothing is
    shared (block ids differ: idle cached blocks go to the bottom of the queue)."""
    rng = np.random.default_rng(seed)
    base = synth.make_workload("mini", 50000, seed, n_requests=40)
    shared = synth.with_shared_prefixes(base, 50000, seed + 10, n_prefixes=3, prefix_len=(16, 70), share=0.8)
    eng = dict(kv_block_size=16, kv_num_blocks=40, max_batch=5, max_prefill_tokens=300, ring_slots=64, eos_token_id=-1)
    tails = list(np.minimum(40, np.cumsum(rng.integers(0, 4, 400))))
    s = Scheduler.from_engine(dict(eng, prefix_cache=True))
    SV.run_schedule(s, shared, lambda pl: [1] * len(pl.sample_seq), tails=tails)
    assert [len(s.outputs[t]) for t in range(40)] == [r["max_new_tokens"] for r in shared]
    assert s.cache_hits > 10 and s.evictions > 0
    s.step(40)
    assert s.committed == 0 and s.pinned == 0 and sorted(s.free) == list(range(40))
    pa, pb = [], []
    a = Scheduler.from_engine(eng)
    SV.run_schedule(a, base, lambda pl: [1] * len(pl.sample_seq), tails=tails, on_plan=pa.append)
    b = Scheduler.from_engine(dict(eng, prefix_cache=True))
    SV.run_schedule(b, base, lambda pl: [1] * len(pl.sample_seq), tails=tails, on_plan=pb.append)
    assert b.cache_hits == 0 and len(pa) == len(pb)
    for x, y in zip(pa, pb):
        for f in ("kind", "tickets", "batch_slots", "input_ids", "positions", "tok_seq", "cu_seqlens", "last_idx", "gen_index", "admitted"):
            assert getattr(x, f) == getattr(y, f), (x.iteration, f)


def test_prefix_cached_service_equals_per_request_generation():
    """The model side: a request whose prompt starts with cached blocks computes only the rest and attends to the shared
    blocks; its stream is exactly what it generates alone. Blocks are matched while their first user is still running,
    after it has retired (idle), and after evictions."""
    cfg = dict(synth.model_config("tiny"), n_layers=2, vocab=97, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96)
    W = M.Weights(cfg, synth.make_weights(cfg, 7, gain_jitter=0.1))
    base = [dict(r, max_new_tokens=min(r["max_new_tokens"], 6)) for r in synth.make_workload("mini", 97, 5, n_requests=14)]
    reqs = synth.with_shared_prefixes(base, 97, 15, n_prefixes=2, prefix_len=(9, 40), share=0.8)
    for i, r in enumerate(reqs):
        if i % 3 == 0:
            r.update(temperature=0.8, top_k=5, top_p=0.9, seed=synth.splitmix64(3, i))
    eng = dict(kv_block_size=4, kv_num_blocks=60, max_batch=3, max_prefill_tokens=120, ring_slots=16, eos_token_id=-1, prefix_cache=True)
    tails = [2, 2, 3, 5, 5, 5, 8, 8, 9, 14]
    ev, sched = SV.serve(cfg, W, eng, reqs, tails=tails)
    assert sched.cache_hits > 8 and sched.evictions > 0
    for t, r in enumerate(reqs):
        assert sched.outputs[t] == SV.generate_reference(cfg, W, r), t


# ---- speculative decoding ----------------------------------------------------------------------------------------------

def _spec_token_fn(sched, f):
    """token_fn for run_schedule: f(ticket, output index) is what the 'model' emits, whatever is fed (rows past a rejected
    draft are computed like the others and ignored by the walk)."""
    def fn(plan):
        if not sched.speculative:
            return [f(t, plan.gen_index[i]) for i, t in enumerate(plan.sample_tickets)]
        return [f(t, plan.gen_index[i] + j) for i, t in enumerate(plan.tickets) for j, _ in enumerate(sched.rows_of(plan, i))]
    return fn


def test_speculative_hand_worked_drafts_acceptance_and_rejection():
    """Prompt 5 6 7 5 6, four tokens wanted, up to three drafts. The model says 7 after the prompt: the last two tokens
    (6, 7) occurred at places 1, 2, so the tokens that followed there (5, 6: two, because only three more tokens may be
    emitted) are fed as drafts behind the 7 at positions 5, 6, 7. Accepting run: the rows say 5, 6, 9: all three emitted.
    Rejecting run: the rows say 5, 8, 9: 5 is emitted and confirms the first draft, 8 is emitted and refutes the second,
    the third row is ignored and the context shrinks by the rejected draft."""
    for rows, outs, ctx in (([5, 6, 9], [7, 5, 6, 9], 8), ([5, 8, 9], [7, 5, 8], 7)):
        s = Scheduler(8, 4, 2, 8192, 8, speculative=3)
        s.submit([5, 6, 7, 5, 6], 4)
        p0 = s.step(1)
        assert (p0.kind, p0.last_idx, p0.row0) == (PREFILL, [4], [0])
        s.commit(p0, [7])
        p1 = s.step(1)
        assert (p1.kind, p1.input_ids, p1.positions, p1.last_idx, p1.row0) == (DECODE, [7, 5, 6], [5, 6, 7], [0, 1, 2], [0])
        assert p1.slot_mapping == [5, 6, 7] and p1.block_tables == [[0, 1]] and p1.seq_lens == [8]
        ev = s.commit(p1, rows)
        s.check_invariants()
        assert s.outputs[0] == outs and s.running[0].ctx_len == ctx and s.running[0].last_token == outs[-1]
        assert [e[1] for e in ev] == list(range(1, len(outs))) and ev[-1][4] == (len(outs) == 4)
        assert (s.drafted, s.accepted) == (2, len(outs) - 2)
    # no earlier occurrence of the last two tokens, a sampled request, or one token left: no drafts
    s = Scheduler(8, 4, 2, 8192, 8, speculative=3)
    s.submit([1, 2, 3, 4, 5], 4)
    s.submit([5, 6, 7, 5, 6], 4, greedy=False)
    s.submit([5, 6, 7, 5, 6], 2)
    p0 = s.step(2)
    s.commit(p0, [9, 7])
    p1 = s.step(2)
    assert p1.input_ids == [9, 7] and p1.last_idx == [0, 1]
    s = Scheduler(8, 4, 2, 8192, 8, speculative=3)
    s.submit([5, 6, 7, 5, 6], 2)
    s.commit(s.step(1), [7])
    assert s.step(1).input_ids == [7]


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_speculative_schedule_emits_what_the_plain_schedule_emits(seed):
    """A 'model' whose token depends on (request, output index) only, with few distinct values so that lookups hit: the
    speculative scheduler emits exactly the plain scheduler's streams in fewer iterations; invariants after every step."""
    f = lambda t, idx: (t * 7 + (idx // 3) * (idx // 3)) % 4
    rng = np.random.default_rng(seed)
    reqs = [dict(prompt=rng.integers(0, 4, int(rng.integers(1, 40))), max_new_tokens=int(rng.integers(1, 30)), temperature=0.0)
            for _ in range(30)]
    for i in (3, 11):
        reqs[i]["temperature"] = 0.7            # sampled requests never speculate
    eng = dict(kv_block_size=4, kv_num_blocks=60, max_batch=4, max_prefill_tokens=64, ring_slots=32, eos_token_id=-1)
    tails = list(np.minimum(30, 1 + np.cumsum(rng.integers(0, 3, 300))))      # (the first poll sees a request: no idle spin)
    a = Scheduler.from_engine(eng)
    SV.run_schedule(a, reqs, _spec_token_fn(a, f), tails=tails)
    b = Scheduler.from_engine(dict(eng, speculative=4))
    seen = []
    SV.run_schedule(b, reqs, _spec_token_fn(b, f), tails=tails, on_plan=seen.append)
    assert [b.outputs[t] for t in range(30)] == [a.outputs[t] for t in range(30)]
    assert b.accepted > 20 and b.drafted > b.accepted and b.iteration < a.iteration
    sampled = {3, 11}
    for pl in seen:
        if pl.kind == DECODE:
            for i, t in enumerate(pl.tickets):
                if t in sampled:
                    assert len(b.rows_of(pl, i)) == 1
    b.step(30)
    assert b.committed == 0 and sorted(b.free) == list(range(60))


def test_speculative_service_equals_per_request_generation():
    """The model side: drafts are fed at consecutive positions of one iteration and every position gets a logits row; what
    is emitted is exactly what the request generates alone, greedy or sampled, and drafts are accepted on the way (a
    random tiny model decoding greedily soon repeats itself)."""
    cfg = dict(synth.model_config("tiny"), n_layers=2, vocab=97, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96)
    W = M.Weights(cfg, synth.make_weights(cfg, 9, gain_jitter=0.1))
    reqs = [dict(r, max_new_tokens=24) for r in synth.make_workload("mini", 97, 5, n_requests=8)]
    reqs[2].update(temperature=0.8, top_k=5, top_p=0.9, seed=synth.splitmix64(3, 2))
    eng = dict(kv_block_size=4, kv_num_blocks=120, max_batch=3, max_prefill_tokens=150, ring_slots=16, eos_token_id=-1, speculative=4)
    ev, sched = SV.serve(cfg, W, eng, reqs)
    assert sched.accepted > 10, (sched.drafted, sched.accepted)
    for t, r in enumerate(reqs):
        assert sched.outputs[t] == SV.generate_reference(cfg, W, r), t
