"""The whole serving loop on the CPU: scheduler + paged forward + sampling. Oracle code: test
infrastructure only.

run_schedule: integer-only run of the scheduler with the token values supplied by a callback
(used alone it gives the schedule; combined with paged_forward it gives the full service).
serve: every request submitted, then iterations until all have finished, in deterministic
mode (everything visible from the first poll) or replaying a recorded sequence of ring tails.
"""
import numpy as np

from . import model as M
from . import sampling as S
from .scheduler import Scheduler, IDLE


def run_schedule(sched, requests, token_fn, tails=None, max_iterations=None, on_plan=None):
    """Submit all requests, then iterate. token_fn(plan) -> list of sampled tokens.
    tails: per non-idle iteration, the ring tail the poll saw (None: all requests visible).
    Returns the list of events (iteration, ticket, index, token, first, last)."""
    for r in requests:
        sched.submit(r["prompt"], r["max_new_tokens"], greedy=r.get("temperature", 0.0) == 0.0)
    events = []
    n = len(requests)
    it = 0
    while max_iterations is None or it < max_iterations:
        tail = n if tails is None else (tails[it] if it < len(tails) else n)
        plan = sched.step(tail)
        sched.check_invariants()
        if plan.kind == IDLE:
            if sched.next_ticket >= n:
                break
            if tails is None or it >= len(tails):
                raise RuntimeError("idle with requests pending: head request can never be admitted")
            continue
        if on_plan is not None:
            on_plan(plan)
        toks = token_fn(plan)
        for ev in sched.commit(plan, toks):
            events.append((plan.iteration,) + ev)
        it += 1
    return events


def serve(cfg, W, eng, requests, tails=None, max_iterations=None, on_plan=None, keep_logits=None):
    """Full service. eng: engine config dict (kv_block_size, kv_num_blocks, max_batch,
    max_prefill_tokens, ring_slots, eos_token_id). Returns (events, scheduler).
    keep_logits: optional list that receives (iteration, logits[n_seq][V]) per iteration."""
    sched = Scheduler.from_engine(eng)
    kv = M.PagedKV(cfg, eng["kv_num_blocks"], eng["kv_block_size"])

    def token_fn(plan):
        logits = M.paged_forward(cfg, W, kv, plan.input_ids, plan.positions, plan.slot_mapping, plan.tok_seq,
                                 plan.block_tables, plan.last_idx)
        if keep_logits is not None:
            keep_logits.append((plan.iteration, logits))
        out = []
        if sched.speculative:           # one token per logits row: row j of a sequence samples output index gen + j
            for i, t in enumerate(plan.tickets):
                r = requests[t]
                for j, row in enumerate(sched.rows_of(plan, i)):
                    out.append(S.sample(logits[row], r["temperature"], r["top_k"], r["top_p"], r["seed"], plan.gen_index[i] + j))
            return out
        for i, t in enumerate(plan.sample_tickets):
            r = requests[t]
            out.append(S.sample(logits[i], r["temperature"], r["top_k"], r["top_p"], r["seed"], plan.gen_index[i]))
        return out

    events = run_schedule(sched, requests, token_fn, tails, max_iterations, on_plan)
    return events, sched


def generate_reference(cfg, W, request, eos=-1):
    """Token stream of one request on its own (contiguous cache): what the service must emit for it
    whatever the batching."""
    m = M.CachedModel(cfg, W)
    logits = m.step(request["prompt"])
    out = []
    for i in range(request["max_new_tokens"]):
        tok = S.sample(logits, request["temperature"], request["top_k"], request["top_p"], request["seed"], i)
        out.append(tok)
        if tok == eos or i + 1 == request["max_new_tokens"]:
            break
        logits = m.step([tok])
    return out
