"""Helpers shared by the GPU parity tests: run a workload on the engine, and check it against the oracle
teacher-forced (the oracle replays the schedule with the engine's own tokens as history, so a legitimate
near-tie cannot make the rest of a stream incomparable)."""
import numpy as np

from oracle import model as M, sampling as S
from oracle.philox import uniform_for_token
from oracle.scheduler import Scheduler
from oracle.serve import run_schedule


def run_engine(B, cfg, eng, blob, reqs, flags=0, window=0, poll_cap=4096, tune=0):
    """Submit everything, run to idle (optionally in windows of `window` iterations), return
    (events, trace, stats)."""
    e = B.Engine(cfg, eng, blob, flags=flags | B.FLAG_TRACE | B.FLAG_EXIT_WHEN_IDLE, tune=tune)
    try:
        for r in reqs:
            e.submit_request(r)
        evs = []
        for _ in range(100000):
            e.run(window)
            e.wait()
            evs.append(e.drain(poll_cap))
            st = e.stats()
            if st["n_running"] == 0 and st["next_ticket"] == len(reqs):
                break
        else:
            raise AssertionError("engine did not drain")
        ev = np.concatenate(evs)
        return ev, e.trace(), e.stats()
    finally:
        e.shutdown()


def event_tuples(ev):
    """(iteration, ticket, index, token, first, last), sorted by (iteration, then order of arrival in the array)."""
    out = [(int(x["iteration"]), int(x["request_id"]), int(x["index"]), int(x["token"]), bool(x["flags"] & 1), bool(x["flags"] & 2))
           for x in ev]
    return out


def check_against_oracle(cfg, W, eng, reqs, ev, trace, rtol, tails=None, tok_rtol=None):
    """Teacher-forced check. Returns dict with counts. Asserts:
    - the schedule (iteration, ticket, index, first/last flags of every event; kind / n_seqs / n_tokens /
      free blocks / admissions of every iteration) is bit-exact;
    - greedy tokens: the engine's token is the oracle's argmax whenever the oracle's top-1 margin exceeds
      2*tol, and within 2*tol of the maximum otherwise (tol = rtol * max|logit| of the row; tok_rtol, when
      given, replaces rtol here: a tighter bound taken from the measured logit error of the kernels);
    - sampled tokens: the engine's token equals the oracle's choice whenever every decision of the sampler
      (top-k membership, top-p cut, CDF bin) is farther than the tolerance from its boundary."""
    gpu = {}
    for x in ev:
        gpu[(int(x["request_id"]), int(x["index"]))] = int(x["token"])
    sched = Scheduler.from_engine(eng)
    kv = M.PagedKV(cfg, eng["kv_num_blocks"], eng["kv_block_size"])
    stats = dict(tokens=0, near_ties=0, greedy_tokens=0, greedy_near_ties=0, sampled_tokens=0, sampled_undecided=0, plans=[])

    def token_fn(plan):
        logits = M.paged_forward(cfg, W, kv, plan.input_ids, plan.positions, plan.slot_mapping, plan.tok_seq,
                                 plan.block_tables, plan.last_idx)
        stats["plans"].append(plan)
        out = []
        for i, t in enumerate(plan.sample_tickets):
            r = reqs[t]
            g = gpu[(t, plan.gen_index[i])]
            row = logits[i]
            tol = (tok_rtol if tok_rtol is not None else rtol) * np.abs(row).max()
            stats["tokens"] += 1
            if r["temperature"] == 0.0:
                order = S.candidate_order(row)
                margin = row[order[0]] - row[order[1]]
                assert row[g] >= row[order[0]] - 2 * tol, (t, plan.gen_index[i], g, int(order[0]), margin, tol)
                stats["greedy_tokens"] += 1
                if margin > 2 * tol:
                    assert g == int(order[0]), (t, plan.gen_index[i], g, int(order[0]), margin, tol)
                else:
                    stats["near_ties"] += 1
                    stats["greedy_near_ties"] += 1
            else:
                u = uniform_for_token(r["seed"], plan.gen_index[i])
                d = S.sample_detail(row, r["temperature"], r["top_k"], r["top_p"], u)
                stats["sampled_tokens"] += 1
                if sampling_decisions_clear(row, r, d, tol):
                    assert g == d["token"], (t, plan.gen_index[i], g, d["token"])
                else:
                    stats["near_ties"] += 1
                    stats["sampled_undecided"] += 1
                    assert sampled_token_plausible(row, r, d, g, tol), (t, plan.gen_index[i], g, d["token"])
            out.append(g)
        return out

    events = run_schedule(sched, reqs, token_fn, tails=tails)
    exp = [(it, t, idx, tok, first, last) for (it, t, idx, tok, first, last) in events]
    got = sorted(event_tuples(ev), key=lambda e: (e[0], next(i for i, b in enumerate(stats["plans"][e[0]].sample_tickets) if b == e[1])))
    assert got == exp
    assert len(trace) == len(stats["plans"])
    for tr, pl in zip(trace, stats["plans"]):
        assert (int(tr["iteration"]), int(tr["kind"]), int(tr["n_seqs"]), int(tr["n_tokens"]), int(tr["free_blocks"]),
                int(tr["n_admitted"])) == (pl.iteration, pl.kind, len(pl.tickets), len(pl.input_ids), pl.free_blocks_after,
                                           len(pl.admitted)), pl.iteration
        if pl.admitted:
            assert int(tr["first_admitted"]) == pl.admitted[0]
        assert (int(tr["n_resumed"]), int(tr["n_preempted"])) == (len(pl.resumed), len(pl.preempted)), pl.iteration
    sched.step(len(reqs))
    stats["sched"] = sched
    return stats


def sampling_decisions_clear(row, r, d, tol):
    """True when logits that differ from `row` by at most tol per element must give the same token.

    With such logits, two candidates can change places only if their logits are within 2 tol of each other. If the
    chosen candidate is farther than that from both of its neighbours in the order (the next one counted even when the
    top-k or top-p cut excludes it), the set of candidates ahead of it is the same on both sides, and so is the set
    behind it up to members near the cuts, whose probabilities are then nearly equal. What is left is arithmetic: each
    probability moves by a relative e^(2 tol / T) - 1 at most, so the top-p cut stays where it is when the cumulative
    mass at the cut and just before it is farther than eps from top_p, and the draw stays in its bin when u * total is
    farther than eps from both edges of the bin."""
    T = r["temperature"]
    order = S.candidate_order(row)
    n = len(d["kept"])
    idx = int(np.nonzero(d["kept"] == d["token"])[0][0])
    near = lambda i, j: abs(row[order[i]] - row[order[j]]) <= 2 * tol
    if (idx > 0 and near(idx - 1, idx)) or (idx + 1 < row.size and near(idx, idx + 1)):
        return False
    eps = np.expm1(2 * tol / T) * 1.5 + 2e-6
    cum = np.cumsum(d["probs"])
    if r["top_p"] < 1.0 and (abs(cum[n - 1] - r["top_p"]) <= eps or (n > 1 and abs(cum[n - 2] - r["top_p"]) <= eps)):
        return False
    lo = d["cdf"][idx - 1] if idx > 0 else -1.0
    if abs(d["cdf"][idx] - d["target"]) <= eps or abs(lo - d["target"]) <= eps:
        return False
    return True


def sampled_token_plausible(row, r, d, g, tol):
    """Necessary condition for token g to be what a correct sampler returns on logits within tol of `row` (used for the
    sampled tokens whose decisions are not clear, instead of skipping them). On such logits the candidates ahead of g
    are those ahead of it in the oracle's order, give or take the candidates within 2 tol of g; every probability moves
    by a relative e^(2 tol / T) - 1 at most; the top-p cut moves by at most the candidates next to it. So the draw
    u * total must fall into g's bin widened by the mass of g's near neighbours and by eps, g's bin must start before
    top_p, and g must be among the top-k or within 2 tol of its boundary."""
    T, top_p = r["temperature"], r["top_p"]
    order = S.candidate_order(row)
    k, n = d["n_topk"], len(d["kept"])
    pos = int(np.nonzero(order == g)[0][0])
    if pos >= k:
        return abs(row[order[k - 1]] - row[g]) <= 2 * tol
    p = d["probs"]
    cum = np.cumsum(p)
    eps = np.expm1(2 * tol / T) * 1.5 + 2e-6
    near = np.abs(row[order[:k]] - row[g]) <= 2 * tol
    m_near = float(p[near].sum() - p[pos])
    lo, hi = (cum[pos - 1] if pos > 0 else 0.0) - m_near - eps, cum[pos] + m_near + eps
    if lo >= top_p:
        return False
    u = d["target"] / d["total"]
    tot_lo, tot_hi = cum[max(n - 2, 0)] - eps, cum[min(n, k - 1)] + eps      # the cut may sit one candidate earlier or later
    return lo <= u * tot_hi and u * tot_lo <= hi


def arithmetic_decided(d, top_p, eps=2e-5):
    """For a sampler that sees the SAME logits as the oracle: candidates are ordered by exact values on both sides, so
    only the fp32 arithmetic of the engine (exponentials, cumulative sums of up to 1024 terms) can move a decision. True
    when the top-p cut and the bin of the draw are farther than eps from their boundaries."""
    n = len(d["kept"])
    cum = np.cumsum(d["probs"])
    if top_p < 1.0 and (abs(cum[n - 1] - top_p) <= eps or (n > 1 and abs(cum[n - 2] - top_p) <= eps)):
        return False          # (top_p = 1 keeps all k candidates on both sides whatever the rounding of the last sum)
    idx = int(np.nonzero(d["kept"] == d["token"])[0][0])
    lo = d["cdf"][idx - 1] if idx > 0 else -1.0
    return abs(d["cdf"][idx] - d["target"]) > eps and abs(lo - d["target"]) > eps


def token_matches_own_logits(row, r, gen_index, token):
    """The engine's token against the oracle's sampler run on the engine's own logits row (float32, widened exactly).
    Greedy: exact. Sampled: exact when arithmetic_decided, else the token must at least be a kept candidate or the next
    one. Returns True when the comparison was exact."""
    row = np.asarray(row, dtype=np.float64)
    if r["temperature"] == 0.0:
        assert token == S.greedy(row), (token, S.greedy(row))
        return True
    d = S.sample_detail(row, r["temperature"], r["top_k"], r["top_p"], uniform_for_token(r["seed"], gen_index))
    if arithmetic_decided(d, r["top_p"]):
        assert token == d["token"], (token, d["token"], gen_index)
        return True
    assert token in set(int(x) for x in S.candidate_order(row)[: len(d["kept"]) + 1])
    return False


ROUTE_MARGIN = 2e-3   # of the largest router logit of the token: beyond it the half-precision logits decide like exact ones


def check_routing(cfg, routing, route_log, stats):
    """The engine's expert selection against the oracle's own (computed on the same history of routings): always k
    distinct experts in range; the same set wherever the oracle's margin between the last selected and the first
    rejected logit is clear of the engine's arithmetic; the same order wherever the selected logits are that far apart."""
    E, k = cfg["n_experts"], cfg["n_active"]
    assert len(route_log) == cfg["n_layers"]
    for rl in route_log:
        sel = routing[rl["layer"]]
        assert sel.shape == rl["own"].shape
        assert sel.max() < E
        assert all(len(set(row)) == k for row in sel.tolist())
        clear = rl["margin"] > ROUTE_MARGIN * rl["scale"]
        stats["pairs"] += len(clear)
        stats["unclear"] += int((~clear).sum())
        same_set = np.sort(sel, axis=1) == np.sort(rl["own"], axis=1)
        assert same_set.all(axis=1)[clear].all(), (rl["layer"], np.nonzero(~same_set.all(axis=1) & clear))
        if "gaps" in rl:
            ordered = clear & (rl["gaps"] > ROUTE_MARGIN * rl["scale"])
            assert (sel == rl["own"])[ordered].all(), rl["layer"]


def check_attention_items(items, plan, whole_contexts):
    """The decode attention's work list against the plan: every 512-token chunk of every decoding sequence's context
    exactly once (as chunks: full ones first; as whole contexts: longest first, the lower batch slot first among equals),
    the fields of an item those of its sequence."""
    items = items.reshape(-1, 8)
    assert plan.kind == 2       # (decode iteration: every sequence that processes one token decodes)
    if whole_contexts is None:  # the scheduler's own choice: told apart by the items unless every context fits one chunk
        if any(r[3] > 0 or r[5] > 1 for r in items.tolist()):
            whole_contexts = False
        elif any(r[1] > 512 for r in items.tolist()):
            whole_contexts = True
        else:
            assert sorted((int(r[2]), 0) for r in items) == sorted((plan.batch_slots[i], 0) for i in range(len(plan.batch_slots))
                                                                   if plan.cu_seqlens[i + 1] - plan.cu_seqlens[i] == 1)
            return None
    
    decoding = [i for i in range(len(plan.batch_slots)) if plan.cu_seqlens[i + 1] - plan.cu_seqlens[i] == 1]
    by_slot = {plan.batch_slots[i]: i for i in decoding}
    seen = set()
    for tok, ctx, bslot, ch, ci, nres, b_end, _ in items.tolist():
        i = by_slot[bslot]
        assert (tok, ctx) == (plan.cu_seqlens[i], plan.seq_lens[i])
        nblocks = -(-ctx // 16)
        if whole_contexts:
            assert (ch, nres, b_end) == (0, 1, nblocks)
            covered = range(0, -(-ctx // 512))
        else:
            assert nres == -(-ctx // 512) and b_end == min(nblocks, 32 * (ch + 1)) and ch < nres
            covered = [ch]
        for k in covered:
            assert (bslot, k) not in seen
            seen.add((bslot, k))
    assert seen == {(plan.batch_slots[i], k) for i in decoding for k in range(-(-plan.seq_lens[i] // 512))}
    if whole_contexts:
        keys = [(-int(r[1]), int(r[2])) for r in items]
        assert keys == sorted(keys)
        assert sorted(int(r[4]) for r in items) == list(range(len(items)))     # one result per sequence
    else:
        full = [int(r[6]) - 32 * int(r[3]) == 32 and int(r[1]) >= 512 * (int(r[3]) + 1) for r in items]
        assert full == sorted(full, reverse=True)                               # the full chunks come first
    return whole_contexts


def stepwise_check(B, cfg, eng, raw, blob, reqs, rtol, max_iters=10000, tune=0, tokens_out=None, item_modes=None):
    """One iteration per blink_run call: batch metadata, block tables and free stack bit-exact against the
    oracle's scheduler; logits within rtol of the row maximum against the oracle's paged forward fed with
    the engine's own token history; every token against the oracle's sampler run on the engine's own logits
    (so sampling is checked exactly, apart from the logit tolerance). Returns the worst relative logit error."""
    W = M.Weights(cfg, raw)
    sched = Scheduler.from_engine(eng)
    kv = M.PagedKV(cfg, eng["kv_num_blocks"], eng["kv_block_size"])
    for r in reqs:
        sched.submit(r["prompt"], r["max_new_tokens"])
    e = B.Engine(cfg, eng, blob, flags=B.FLAG_TRACE | B.FLAG_EXIT_WHEN_IDLE | B.FLAG_KEEP_LOGITS, tune=tune)
    D = B.DBG
    worst = 0.0
    moe_stats = dict(pairs=0, unclear=0)
    try:
        for r in reqs:
            e.submit_request(r)
        for it in range(max_iters):
            e.run(1)
            e.wait()
            plan = sched.step(len(reqs))
            sched.check_invariants()
            if eng.get("prefix_cache"):
                st = e.stats()
                assert (st["prefix_hit_blocks"], st["prefix_evictions"], st["pinned_blocks"], st["committed_blocks"]) == \
                    (sched.cache_hits, sched.evictions, sched.pinned, sched.committed), (it, st)
            if plan.kind == 0:
                assert e.stats()["iterations"] == it
                assert moe_stats["unclear"] <= 0.08 * moe_stats["pairs"], moe_stats
                return worst
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
            if cfg["dtype"] == 1 and plan.kind == 2:
                forced = False if tune & 0x808000 else True if tune & 0x400080 else None   # bit 7: the chain without merge kernels
                mode = check_attention_items(e.debug_read(D.ATTN_ITEMS, np.uint32), plan, forced)
                if item_modes is not None:
                    item_modes.append(mode)
            routing, route_log = None, None
            if cfg.get("n_experts", 0):   # mixture of experts: the oracle follows the engine's routing and reports its own
                routing = e.debug_read(D.ROUTING, np.uint32).reshape(cfg["n_layers"], len(plan.input_ids), cfg["n_active"])
                route_log = []
            ref = M.paged_forward(cfg, W, kv, plan.input_ids, plan.positions, plan.slot_mapping, plan.tok_seq,
                                  plan.block_tables, plan.last_idx, routing=routing, route_log=route_log)
            if routing is not None:
                check_routing(cfg, routing, route_log, moe_stats)
            evs = e.drain()
            by_ticket = {int(x["request_id"]): int(x["token"]) for x in evs}
            assert sorted(by_ticket) == sorted(plan.sample_tickets)
            if plan.sample_seq:
                got = e.debug_read(D.LOGITS, np.float32).reshape(len(plan.sample_seq), cfg["vocab"])
                err = np.abs(got - ref).max(axis=1) / np.abs(ref).max(axis=1)
                worst = max(worst, float(err.max()))
                assert err.max() < rtol, (it, err)
                for i, t in enumerate(plan.sample_tickets):
                    token_matches_own_logits(got[i], reqs[t], plan.gen_index[i], by_ticket[t])
            if tokens_out is not None:
                for t in plan.sample_tickets:
                    tokens_out.setdefault(t, []).append(by_ticket[t])
            sched.commit(plan, [by_ticket[t] for t in plan.sample_tickets])   # the engine's tokens are the history
        raise AssertionError("did not finish")
    finally:
        e.shutdown()


def stepwise_check_speculative(B, cfg, eng, raw, blob, reqs, rtol, max_iters=10000, tune=0):
    """Speculative decoding, one iteration per blink_run call: the drafts (input ids behind each last token), positions,
    slot mapping, block tables, free stack and the logits rows' token indices bit-exact against the oracle's scheduler;
    every logits row (one per fed position) within rtol of the oracle's paged forward on the engine's token history; the
    verification walk exact: the oracle commits, row by row, its own sampler's tokens on the engine's logits rows, and
    the events it emits (request, index, token, first/last) must be the engine's events of the iteration, the counters of
    drafted and accepted tokens the engine's counters. Returns (worst relative logit error, tokens per ticket)."""
    W = M.Weights(cfg, raw)
    sched = Scheduler.from_engine(eng)
    assert sched.speculative
    kv = M.PagedKV(cfg, eng["kv_num_blocks"], eng["kv_block_size"])
    for r in reqs:
        sched.submit(r["prompt"], r["max_new_tokens"], greedy=r["temperature"] == 0.0)
    e = B.Engine(cfg, eng, blob, flags=B.FLAG_TRACE | B.FLAG_EXIT_WHEN_IDLE | B.FLAG_KEEP_LOGITS, tune=tune)
    D = B.DBG
    worst = 0.0
    toks = {}
    moe_stats = dict(pairs=0, unclear=0)
    try:
        for r in reqs:
            e.submit_request(r)
        for it in range(max_iters):
            e.run(1)
            e.wait()
            plan = sched.step(len(reqs))
            sched.check_invariants()
            if plan.kind == 0:
                st = e.stats()
                assert st["iterations"] == it
                assert moe_stats["unclear"] <= 0.08 * moe_stats["pairs"], moe_stats
                assert (st["spec_drafted"], st["spec_accepted"]) == (sched.drafted, sched.accepted)
                assert st["tokens_out"] == sum(len(v) for v in toks.values())
                assert st["free_blocks"] == eng["kv_num_blocks"] and st["committed_blocks"] == 0
                return worst, toks
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
            routing, route_log = None, None
            if cfg.get("n_experts", 0):   # mixture of experts: the oracle follows the engine's routing and reports its own
                routing = e.debug_read(D.ROUTING, np.uint32).reshape(cfg["n_layers"], len(plan.input_ids), cfg["n_active"])
                route_log = []
            ref = M.paged_forward(cfg, W, kv, plan.input_ids, plan.positions, plan.slot_mapping, plan.tok_seq,
                                  plan.block_tables, plan.last_idx, routing=routing, route_log=route_log)
            if routing is not None:
                check_routing(cfg, routing, route_log, moe_stats)
            got = e.debug_read(D.LOGITS, np.float32).reshape(len(plan.last_idx), cfg["vocab"])
            err = np.abs(got - ref).max(axis=1) / np.abs(ref).max(axis=1)
            worst = max(worst, float(err.max()))
            assert err.max() < rtol, (it, err)
            evs = e.drain()
            mine = {}
            for x in evs:
                mine.setdefault(int(x["request_id"]), []).append((int(x["index"]), int(x["token"]), bool(x["flags"] & 1), bool(x["flags"] & 2)))
            row_tokens = []
            for i, t in enumerate(plan.tickets):
                r = reqs[t]
                rows = sched.rows_of(plan, i)
                if r["temperature"] == 0.0:
                    row_tokens += [S.greedy(np.asarray(got[row], dtype=np.float64)) for row in rows]
                else:           # a sampled request has one row; its token is checked against the oracle's sampler on that row
                    assert len(rows) == 1 and len(mine[t]) == 1
                    token_matches_own_logits(got[rows[0]], r, plan.gen_index[i], mine[t][0][1])
                    row_tokens.append(mine[t][0][1])
            exp = {}
            for (t, idx, tok, first, last) in sched.commit(plan, row_tokens):
                exp.setdefault(t, []).append((idx, tok, first, last))
                toks.setdefault(t, []).append(tok)
            assert {t: sorted(v) for t, v in mine.items()} == exp, (it, mine, exp)
            assert all(int(x["iteration"]) == plan.iteration for x in evs)
        raise AssertionError("did not finish")
    finally:
        e.shutdown()
