"""GPU parity of prefix caching: the scheduler's matches, reference counts, free queue and evictions bit-exact against
the oracle's after every iteration (block tables, slot mapping, free queue, counters), the logits of prompts that start
behind a cached prefix within the stated tolerance, every token against the oracle's sampler on the engine's own logits."""
import numpy as np
import pytest

import synth
from tests import parity
from tests.test_gpu_parity import setup, sampled
from tests.test_gpu_moe import free_run_tokens

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,dtype,seed", [("mini_gqa", 1, 151), ("mini_gqa128", 1, 152), ("mini_gqa", 0, 153)])
def test_prefix_cache_stepwise(lib, name, dtype, seed):
    """The mini request mix with three common prompt heads of 16..70 tokens behind a pool small enough that idle cached
    blocks are evicted: matches on blocks in use, on idle blocks, and after evictions."""
    cfg, eng, raw, blob = setup(name, seed)
    if dtype == 0:
        cfg = dict(cfg, dtype=0)
        raw = synth.make_weights(cfg, seed, gain_jitter=0.1)
        blob = synth.pack_blob(cfg, raw)
    eng = dict(eng, prefix_cache=True, kv_num_blocks=24, max_batch=5, ring_slots=32)
    base = synth.make_workload("mini", cfg["vocab"], seed + 100, n_requests=26)
    reqs = sampled(synth.with_shared_prefixes(base, cfg["vocab"], seed + 200, n_prefixes=3, prefix_len=(16, 70), share=0.8), seed)
    toks = {}
    worst = parity.stepwise_check(lib, cfg, eng, raw, blob, reqs, rtol=2e-2 if dtype else 2e-4, tokens_out=toks)
    print(name, "dtype", dtype, "worst relative logit error", worst)
    # the free-running loop makes the same tokens and ends with every block free and nothing pinned
    e = lib.Engine(cfg, eng, blob, flags=lib.FLAG_EXIT_WHEN_IDLE)
    try:
        for r in reqs:
            e.submit_request(r)
        e.run(0)
        e.wait()
        ev = e.drain(1 << 16)
        st = e.stats()
    finally:
        e.shutdown()
    got = {}
    for rid, idx, tok in sorted((int(x["request_id"]), int(x["index"]), int(x["token"])) for x in ev):
        got.setdefault(rid, []).append(tok)
    assert got == toks
    assert st["free_blocks"] == eng["kv_num_blocks"] and st["pinned_blocks"] == 0 and st["committed_blocks"] == 0
    assert st["prefix_hit_blocks"] > 10 and st["prefix_evictions"] > 0


@pytest.mark.parametrize("tune", [0, 0x400000])    # bit 22: the decode attention takes whole contexts (here one of 4200 tokens, nine rounds)
def test_prefix_cache_long_prefix_over_256_blocks(lib, tune):
    """A prompt head of 4200 tokens (262 blocks: more than the scheduler's 256 threads take in one strip) shared by three
    requests: the second matches it while the first is running, both retire (262 blocks go idle), the third matches
    the idle blocks; a fourth, unrelated prompt then evicts part of the head."""
    cfg, eng, raw, blob = setup("mini_gqa", 154)
    eng = dict(eng, prefix_cache=True, kv_num_blocks=300, max_batch=1, max_seq_len=4400, max_prefill_tokens=4400, ring_slots=8)
    rng = np.random.default_rng(154)
    head = rng.integers(0, cfg["vocab"], 4200).astype(np.int32)
    def rq(tail_len, own_seed, n):
        own = np.random.default_rng(own_seed).integers(0, cfg["vocab"], tail_len).astype(np.int32)
        return dict(arrival_s=0.0, prompt=np.concatenate([head, own]).astype(np.int32), max_new_tokens=n, temperature=0.0, top_k=0, top_p=1.0, seed=0)
    fresh = dict(arrival_s=0.0, prompt=rng.integers(0, cfg["vocab"], 1500).astype(np.int32), max_new_tokens=2, temperature=0.0, top_k=0, top_p=1.0, seed=0)
    reqs = [rq(5, 1, 3), rq(40, 2, 2), fresh, rq(17, 3, 2)]
    worst = parity.stepwise_check(lib, cfg, eng, raw, blob, reqs, rtol=2e-2, tune=tune)
    print("long shared head, tune", hex(tune), ": worst relative logit error", worst)


def test_prefix_cache_batch_shares_head_in_use(lib):
    """max_batch 4: requests that share a head run side by side (reference counts above one), retire in different
    iterations, and new arrivals match blocks that are still in use."""
    cfg, eng, raw, blob = setup("mini_gqa128", 155)
    eng = dict(eng, prefix_cache=True, kv_num_blocks=64, max_batch=4)
    rng = np.random.default_rng(155)
    head = rng.integers(0, cfg["vocab"], 70).astype(np.int32)
    reqs = []
    for i in range(12):
        own = rng.integers(0, cfg["vocab"], int(rng.integers(1, 40))).astype(np.int32)
        reqs.append(dict(arrival_s=0.0, prompt=np.concatenate([head[: 70 if i % 3 else 33], own]).astype(np.int32),
                         max_new_tokens=int(rng.integers(1, 9)), temperature=0.0, top_k=0, top_p=1.0, seed=i))
    worst = parity.stepwise_check(lib, cfg, eng, raw, blob, reqs, rtol=2e-2)
    print("shared head in use: worst relative logit error", worst)


def test_prefix_cache_rejected_with_other_modes(lib):
    cfg, eng, raw, blob = setup("mini_gqa", 156)
    for other in ("chunked_prefill", "preemption"):
        with pytest.raises(lib.BlinkError):
            lib.Engine(cfg, dict(eng, prefix_cache=True, **{other: True}), blob)
