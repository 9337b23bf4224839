"""GPU parity of speculative decoding: drafts by lookup in the request's own tokens, a logits row per fed position,
row-by-row verification. The scheduler's metadata (drafts included) bit-exact against the oracle's after every iteration,
every logits row within the stated tolerance, the emitted tokens exactly those of the oracle's walk over the engine's own
logits rows, the counters of drafted and accepted tokens equal."""
import numpy as np
import pytest

import synth
from tests import parity
from tests.test_gpu_parity import setup

pytestmark = pytest.mark.gpu


def repetitive_requests(cfg, eng, seed, n_requests, max_new=40):
    reqs = synth.with_repetition(synth.make_workload("mini", cfg["vocab"], seed + 100, n_requests=n_requests), cfg["vocab"], seed + 200)
    for i, r in enumerate(reqs):
        r["max_new_tokens"] = max(1, min(max_new if i % 4 else 3, eng["max_seq_len"] - len(r["prompt"]) - 1))
    return reqs


def free_run(lib, cfg, eng, blob, reqs):
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
    return got, st


@pytest.mark.parametrize("name,dtype,seed,k", [("mini_gqa", 1, 161, 4), ("mini_gqa128", 1, 162, 7), ("mini_gqa", 0, 163, 3), ("mini_g8", 1, 164, 2),
                                               ("mini_moe", 1, 170, 3)])
def test_speculative_stepwise(lib, name, dtype, seed, k):
    """Prompts that repeat a short phrase, so that lookups hit from the first decode iteration on, and a random model that
    decodes greedily and soon repeats itself, so that drafts are accepted as well as rejected; every third request samples
    (and must never speculate); some requests want three tokens only (drafts cut to what may still be emitted)."""
    cfg, eng, raw, blob = setup(name, seed)
    if dtype == 0:
        cfg = dict(cfg, dtype=0)
        raw = synth.make_weights(cfg, seed, gain_jitter=0.1)
        blob = synth.pack_blob(cfg, raw)
    eng = dict(eng, speculative=k)
    reqs = repetitive_requests(cfg, eng, seed, 11)
    for i in range(2, len(reqs), 3):
        reqs[i].update(temperature=0.8, top_k=50, top_p=0.9, seed=synth.splitmix64(seed, i))
    worst, toks = parity.stepwise_check_speculative(lib, cfg, eng, raw, blob, reqs, rtol=2e-2 if dtype else 2e-4)
    got, st = free_run(lib, cfg, eng, blob, reqs)
    print(name, "dtype", dtype, "k", k, "worst relative logit error", worst, "drafted", st["spec_drafted"], "accepted", st["spec_accepted"],
          "iterations", st["iterations"])
    assert got == toks                                     # the free-running loop emits the same streams
    assert st["spec_accepted"] > 20 and st["spec_drafted"] > st["spec_accepted"]
    assert st["free_blocks"] == eng["kv_num_blocks"] and st["committed_blocks"] == 0


def test_speculative_streams_equal_plain_streams_fp32(lib):
    """fp32 model, greedy requests: the speculative engine emits token for token what the plain engine emits (the logits
    of the two differ by rounding order only, far below the margins of this model), in fewer iterations."""
    cfg, eng, raw, blob = setup("mini_gqa", 165)
    cfg = dict(cfg, dtype=0)
    raw = synth.make_weights(cfg, 165, gain_jitter=0.1)
    blob = synth.pack_blob(cfg, raw)
    reqs = repetitive_requests(cfg, eng, 165, 14)
    plain, st0 = free_run(lib, cfg, eng, blob, reqs)
    spec, st1 = free_run(lib, cfg, dict(eng, speculative=5), blob, reqs)
    assert spec == plain
    assert st1["iterations"] < st0["iterations"] and st1["tokens_out"] == st0["tokens_out"] == sum(len(v) for v in plain.values())
    print("iterations", st0["iterations"], "->", st1["iterations"], "drafted", st1["spec_drafted"], "accepted", st1["spec_accepted"])


@pytest.mark.parametrize("tune", [0, 0x400000])    # bit 22: the decode attention takes whole contexts, as it does by itself with many sequences
def test_speculative_wide_batch_and_long_lookback(lib, tune):
    """40 batch slots with up to 8 fed tokens each (a decode iteration of several hundred tokens: the tiled GEMM schedules
    and query tiles of many sequences in one launch), prompts of up to 1500 tokens (lookups past the 1024-position window
    must not be found; contexts of several attention chunks)."""
    cfg, eng, raw, blob = setup("mini_g6", 166)
    eng = dict(eng, speculative=7, max_batch=40, kv_num_blocks=1200, max_seq_len=1600, max_prefill_tokens=2000, ring_slots=64)
    rng = np.random.default_rng(166)
    reqs = []
    for i in range(44):
        n = int(rng.integers(1100, 1500)) if i % 11 == 0 else int(rng.integers(3, 90))
        if i % 11 == 0:      # a phrase at the very start only, then tokens that never repeat: the last bigram lies out of the window
            p = np.concatenate([np.resize(rng.integers(0, 50, 3), 30), 50 + rng.permutation(cfg["vocab"] - 50)[: n - 30]])
        else:
            p = np.resize(rng.integers(0, cfg["vocab"], int(rng.integers(2, 6))), n)
        reqs.append(dict(arrival_s=0.0, prompt=p.astype(np.int32), max_new_tokens=int(rng.integers(1, 14)), temperature=0.0, top_k=0, top_p=1.0, seed=i))
    worst, toks = parity.stepwise_check_speculative(lib, cfg, eng, raw, blob, reqs, rtol=2e-2, tune=tune)
    print("wide speculative batch, tune", hex(tune), ": worst relative logit error", worst)


def test_speculative_rejected_with_other_modes_and_bad_counts(lib):
    cfg, eng, raw, blob = setup("mini_gqa", 167)
    for other in ("chunked_prefill", "preemption", "prefix_cache"):
        with pytest.raises(lib.BlinkError):
            lib.Engine(cfg, dict(eng, speculative=3, **{other: True}), blob)
    with pytest.raises(lib.BlinkError):
        lib.Engine(cfg, dict(eng, speculative=8), blob)


def test_speculative_lookup_window_boundary(lib):
    """A model whose attention output and FFN down projections are zero emits f(last token) whatever the context, so the
    test can plant the bigram (last prompt token, first output) at the start of a prompt: with a prompt of 1025 tokens it
    lies at the far edge of the 1024-position window and its continuation is drafted (and accepted: it is f of the first
    output); with 1026 tokens it lies one position outside and nothing is drafted. Both against the oracle, bit-exact."""
    from oracle import model as M
    cfg, eng, raw, blob = setup("mini_gqa128", 168)
    for l in range(cfg["n_layers"]):
        raw[f"l{l}.wo"] = np.zeros_like(raw[f"l{l}.wo"])
        raw[f"l{l}.wd"] = np.zeros_like(raw[f"l{l}.wd"])
    blob = synth.pack_blob(cfg, raw)
    W = M.Weights(cfg, raw)
    f = {}
    def nxt(a):       # the oracle's f, with its margin relative to the largest logit
        if a not in f:
            row = M.CachedModel(cfg, W).step([a])
            o = np.argsort(-row)
            f[a] = (int(o[0]), float((row[o[0]] - row[o[1]]) / np.abs(row).max()))
        return f[a]
    a = next(t for t in range(cfg["vocab"]) if nxt(t)[1] > 0.05 and nxt(nxt(t)[0])[1] > 0.05 and nxt(t)[0] != t)
    x0, x1 = nxt(a)[0], nxt(nxt(a)[0])[0]
    eng = dict(eng, speculative=3, max_batch=2, kv_num_blocks=140, max_seq_len=1100, max_prefill_tokens=2200, ring_slots=8)
    rng = np.random.default_rng(168)
    pool = np.array([t for t in rng.permutation(cfg["vocab"]) if t not in (a, x0)])
    reqs = []
    for P in (1025, 1026):
        p = np.concatenate([[a, x0, x1], pool[: P - 4], [a]]).astype(np.int32)
        assert len(p) == P
        reqs.append(dict(arrival_s=0.0, prompt=p, max_new_tokens=5, temperature=0.0, top_k=0, top_p=1.0, seed=0))
    seen = {}
    for i, r in enumerate(reqs):       # one request at a time: the first decode iteration of each is the case
        e = lib.Engine(cfg, eng, blob, flags=lib.FLAG_EXIT_WHEN_IDLE)
        try:
            e.submit_request(r)
            e.run(2)
            e.wait()
            seen[i] = list(e.debug_read(lib.DBG.INPUT_IDS, np.int32))
        finally:
            e.shutdown()
    assert seen[0][:2] == [x0, x1] and len(seen[0]) >= 2        # drafted from the edge of the window
    assert seen[1] == [x0]                                      # one position further back: not found
    parity.stepwise_check_speculative(lib, cfg, eng, raw, blob, reqs, rtol=2e-2)


def test_speculative_windows_give_the_same_streams(lib):
    """The same speculative run in windows of 2 iterations (blink_run(2) again and again: the drafts of an iteration are
    looked up from what the previous window published) and in one go: identical events."""
    cfg, eng, raw, blob = setup("mini_gqa", 169)
    eng = dict(eng, speculative=4)
    reqs = repetitive_requests(cfg, eng, 169, 10)
    ev1, tr1, st1 = parity.run_engine(lib, cfg, eng, blob, reqs)
    ev2, tr2, st2 = parity.run_engine(lib, cfg, eng, blob, reqs, window=2)
    key = lambda ev: sorted((int(x["request_id"]), int(x["index"]), int(x["token"]), int(x["iteration"]), int(x["flags"])) for x in ev)
    assert key(ev1) == key(ev2)
    assert (st1["spec_drafted"], st1["spec_accepted"], st1["iterations"]) == (st2["spec_drafted"], st2["spec_accepted"], st2["iterations"])
    assert st1["spec_accepted"] > 10


def test_speculative_end_of_sequence_inside_a_run_of_drafts(lib):
    """The end-of-sequence token set to a token the streams emit often: a request finishes at the row that emits it, whether
    the drafts behind it would have been confirmed or not, and the rows behind it are ignored."""
    from collections import Counter
    cfg, eng, raw, blob = setup("mini_gqa", 171)
    eng = dict(eng, speculative=4)
    reqs = repetitive_requests(cfg, eng, 171, 10)
    _, toks = parity.stepwise_check_speculative(lib, cfg, eng, raw, blob, reqs, rtol=2e-2)
    late = Counter(t for v in toks.values() for t in v[3:])
    eos = late.most_common(1)[0][0]
    eng2 = dict(eng, eos_token_id=int(eos))
    _, toks2 = parity.stepwise_check_speculative(lib, cfg, eng2, raw, blob, reqs, rtol=2e-2)
    cut = sum(1 for t, v in toks2.items() if v[-1] == eos and len(v) < len(toks[t]))
    assert cut >= 1, (eos, cut)
    for t, v in toks2.items():
        assert eos not in v[:-1]
