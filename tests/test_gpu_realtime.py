"""Requests arriving while the loop runs: a producer thread writes the ring, the main thread reads tokens, the
device admits whatever it sees. The schedule depends on timing, so the oracle replays it from the recorded ring
tails (one per iteration) and must reproduce every admission, batch slot, block id and token count; token
streams are checked teacher-forced as elsewhere."""
import threading
import time

import numpy as np
import pytest

import synth
from oracle import model as M
from tests import parity

pytestmark = pytest.mark.gpu


def test_arrivals_during_the_loop_replay_against_oracle(lib):
    cfg, eng = synth.model_config("mini_gqa"), synth.engine_config("mini_gqa")
    eng = dict(eng, ring_slots=8)                         # smaller than the request count: slots are reused
    raw = synth.make_weights(cfg, 77, gain_jitter=0.1)
    blob = synth.pack_blob(cfg, raw)
    reqs = synth.make_workload("mini", cfg["vocab"], 177, n_requests=30)
    for i, r in enumerate(reqs):
        r["max_new_tokens"] = min(r["max_new_tokens"], 12)
        if i % 3 == 0:
            r.update(temperature=0.8, top_k=40, top_p=0.9, seed=synth.splitmix64(5, i))
    e = lib.Engine(cfg, eng, blob, flags=lib.FLAG_TRACE)
    rng = np.random.default_rng(3)
    gaps = rng.exponential(0.002, len(reqs))
    full_hits = [0]

    def producer():
        for r, g in zip(reqs, gaps):
            time.sleep(float(g))
            while True:
                try:
                    e.submit_request(r)
                    break
                except lib.BlinkError as ex:
                    assert ex.code == lib.ERR_FULL
                    full_hits[0] += 1
                    time.sleep(0.0005)

    try:
        e.run(0)                                          # until stopped
        th = threading.Thread(target=producer)
        th.start()
        evs, done = [], 0
        deadline = time.time() + 60
        while done < len(reqs) and time.time() < deadline:
            ev = e.poll()
            if ev.size:
                evs.append(ev.copy())
                done += int(np.count_nonzero(ev["flags"] & 2))
            else:
                time.sleep(0.0002)
        th.join()
        e.stop()
        assert done == len(reqs)
        ev = np.concatenate(evs)
        trace = e.trace()
        st = e.stats()
    finally:
        e.shutdown()
    assert st["free_blocks"] == eng["kv_num_blocks"] and st["n_running"] == 0
    tails = [int(t) for t in trace["tail"]]
    assert tails == sorted(tails) and tails[-1] <= len(reqs)
    res = parity.check_against_oracle(cfg, M.Weights(cfg, raw), eng, reqs, ev, trace, rtol=2e-2, tails=tails, tok_rtol=2e-3)
    # per request: consecutive indices, device timestamps increasing
    for t in range(len(reqs)):
        mine = ev[ev["request_id"] == t]
        assert list(mine["index"]) == list(range(reqs[t]["max_new_tokens"]))
        assert np.all(np.diff(mine["device_ns"].astype(np.int64)) > 0)
    print("real-time: iterations", len(trace), "distinct tails", len(set(tails)), "ring-full retries", full_hits[0],
          "greedy near ties", res["greedy_near_ties"], "of", res["greedy_tokens"], "sampled undecided", res["sampled_undecided"], "of",
          res["sampled_tokens"])
    assert len(set(tails)) > 3
    # (every sampled token that is not decided has passed the plausibility check of its CDF bin instead)
    assert res["greedy_near_ties"] <= max(2, res["greedy_tokens"] // 8)
