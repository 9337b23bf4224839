"""Helpers shared by the GPU parity tests: run a workload on the engine, and check it against the oracle
teacher-forced (the oracle replays the schedule with the engine's own tokens as history, so a legitimate
near-tie cannot make the rest of a stream incomparable)."""
import numpy as np

from oracle import model as M, sampling as S
from oracle.philox import uniform_for_token
from oracle.scheduler import Scheduler
from oracle.serve import run_schedule


def run_engine(B, cfg, eng, blob, reqs, flags=0, window=0, poll_cap=4096):
    """Submit everything, run to idle (optionally in windows of `window` iterations), return
    (events, trace, stats)."""
    e = B.Engine(cfg, eng, blob, flags=flags | B.FLAG_TRACE | B.FLAG_EXIT_WHEN_IDLE)
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


def check_against_oracle(cfg, W, eng, reqs, ev, trace, rtol, tails=None):
    """Teacher-forced check. Returns dict with counts. Asserts:
    - the schedule (iteration, ticket, index, first/last flags of every event; kind / n_seqs / n_tokens /
      free blocks / admissions of every iteration) is bit-exact;
    - greedy tokens: the engine's token is the oracle's argmax whenever the oracle's top-1 margin exceeds
      2*tol, and within 2*tol of the maximum otherwise (tol = rtol * max|logit| of the row);
    - sampled tokens: the engine's token equals the oracle's choice whenever every decision of the sampler
      (top-k membership, top-p cut, CDF bin) is farther than the tolerance from its boundary."""
    gpu = {}
    for x in ev:
        gpu[(int(x["request_id"]), int(x["index"]))] = int(x["token"])
    sched = Scheduler(eng["kv_num_blocks"], eng["kv_block_size"], eng["max_batch"], eng["max_prefill_tokens"],
                      eng["ring_slots"], eng.get("eos_token_id", -1))
    kv = M.PagedKV(cfg, eng["kv_num_blocks"], eng["kv_block_size"])
    stats = dict(tokens=0, near_ties=0, plans=[])

    def token_fn(plan):
        logits = M.paged_forward(cfg, W, kv, plan.input_ids, plan.positions, plan.slot_mapping, plan.tok_seq,
                                 plan.block_tables, plan.last_idx)
        stats["plans"].append(plan)
        out = []
        for i, t in enumerate(plan.tickets):
            r = reqs[t]
            g = gpu[(t, plan.gen_index[i])]
            row = logits[i]
            tol = rtol * np.abs(row).max()
            stats["tokens"] += 1
            if r["temperature"] == 0.0:
                order = S.candidate_order(row)
                margin = row[order[0]] - row[order[1]]
                assert row[g] >= row[order[0]] - 2 * tol, (t, plan.gen_index[i], g, int(order[0]), margin, tol)
                if margin > 2 * tol:
                    assert g == int(order[0]), (t, plan.gen_index[i], g, int(order[0]), margin, tol)
                else:
                    stats["near_ties"] += 1
            else:
                u = uniform_for_token(r["seed"], plan.gen_index[i])
                d = S.sample_detail(row, r["temperature"], r["top_k"], r["top_p"], u)
                if sampling_decisions_clear(row, r, d, tol):
                    assert g == d["token"], (t, plan.gen_index[i], g, d["token"])
                else:
                    stats["near_ties"] += 1
                    assert g in set(int(x) for x in S.candidate_order(row)[: d["n_topk"] + 1])
            out.append(g)
        return out

    events = run_schedule(sched, reqs, token_fn, tails=tails)
    exp = [(it, t, idx, tok, first, last) for (it, t, idx, tok, first, last) in events]
    got = sorted(event_tuples(ev), key=lambda e: (e[0], next(i for i, b in enumerate(stats["plans"][e[0]].tickets) if b == e[1])))
    assert got == exp
    assert len(trace) == len(stats["plans"])
    for tr, pl in zip(trace, stats["plans"]):
        assert (int(tr["iteration"]), int(tr["kind"]), int(tr["n_seqs"]), int(tr["n_tokens"]), int(tr["free_blocks"]),
                int(tr["n_admitted"])) == (pl.iteration, pl.kind, len(pl.tickets), len(pl.input_ids), pl.free_blocks_after,
                                           len(pl.admitted)), pl.iteration
        if pl.admitted:
            assert int(tr["first_admitted"]) == pl.admitted[0]
    sched.step(len(reqs))
    stats["sched"] = sched
    return stats


def sampling_decisions_clear(row, r, d, tol):
    """True when no decision of the sampler is within the logit tolerance of flipping."""
    T = r["temperature"]
    order = S.candidate_order(row)
    k = d["n_topk"]
    if k < row.size and row[order[k - 1]] - row[order[k]] <= 2 * tol:
        return False                      # top-k membership is a near-tie
    # a logit error of tol changes each kept probability by a relative e^(2 tol/T) - 1 at most
    eps = np.expm1(2 * tol / T) * 2 + 1e-5
    p = d["probs"]
    cum = np.cumsum(p)
    n = len(d["kept"])
    if abs(cum[n - 1] - r["top_p"]) <= eps or (n > 1 and abs(cum[n - 2] - r["top_p"]) <= eps):
        return False                      # the top-p cut is near a boundary
    # candidates must keep their order (else the CDF is permuted)
    z = row[order[: n + 1]] if n < row.size else row[order[:n]]
    if np.any(np.diff(z) > -2 * tol) and n > 1:
        gaps = -np.diff(row[order[:n]])
        if np.any(gaps <= 2 * tol):
            return False
    target = d["target"]
    if np.any(np.abs(d["cdf"] - target) <= eps * max(1.0, d["total"])):
        return False                      # the draw lands near a CDF boundary
    return True
