"""Seeded request workloads shaped like the five configurations.

A request is a dict: arrival_s (float), prompt (int32 array), max_new_tokens (int),
temperature (float, 0 = greedy), top_k (int, 0 = all), top_p (float), seed (uint64 as int).
"""
import numpy as np

_M64 = (1 << 64) - 1


def splitmix64(seed, index):
    """Per-request sampling seed: the splitmix64 output function applied to seed + (index+1)*golden."""
    z = (seed + (index + 1) * 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def _lognormal_len(rng, n, median, sigma, cap):
    x = rng.lognormal(np.log(median), sigma, n)
    return np.clip(np.rint(x), 1, cap).astype(np.int64)


def make_workload(name, vocab, seed, n_requests=None, rate=None):
    """Returns a list of request dicts sorted by arrival time (ticket order = list order)."""
    rng = np.random.default_rng(seed)
    greedy = dict(temperature=0.0, top_k=0, top_p=1.0)
    if name == "tiny":
        n = n_requests or 8
        plen = rng.integers(16, 65, n)
        olen = np.full(n, 32)
        arr = np.zeros(n)
        samp = greedy
    elif name == "churn":
        n = n_requests or 256
        arr = np.cumsum(rng.exponential(1.0 / (rate or 20.0), n))
        plen = _lognormal_len(rng, n, 256, 0.8, 2048)
        olen = rng.integers(64, 257, n)
        samp = greedy
    elif name == "llama3_8b":
        n = n_requests or 1024
        arr = np.cumsum(rng.exponential(1.0 / (rate or 8.0), n))
        plen = _lognormal_len(rng, n, 512, 1.0, 4096)
        olen = _lognormal_len(rng, n, 128, 0.7, 1024)
        samp = dict(temperature=0.8, top_k=50, top_p=0.9)
    elif name == "sched_stress":
        n = n_requests or 4096
        arr = (np.arange(n) // 512) * 0.050
        plen = rng.integers(4, 33, n)
        olen = rng.integers(1, 17, n)
        samp = greedy
    elif name == "mini":  # parity-test mix: ragged prompts around block and tile boundaries
        n = n_requests or 10
        arr = np.zeros(n)
        plen = rng.integers(1, 100, n)
        plen[: min(n, 5)] = np.array([1, 15, 16, 17, 64])[: min(n, 5)]
        olen = rng.integers(1, 40, n)
        samp = greedy
    else:
        raise ValueError(name)
    reqs = []
    for i in range(n):
        reqs.append(dict(arrival_s=float(arr[i]),
                         prompt=rng.integers(0, vocab, int(plen[i])).astype(np.int32),
                         max_new_tokens=int(olen[i]), seed=splitmix64(seed, i), **samp))
    return reqs


def with_shared_prefixes(reqs, vocab, seed, n_prefixes=4, prefix_len=(16, 200), share=0.75):
    """A copy of the request list in which a fraction `share` of the requests start with one of `n_prefixes` common
    token sequences (system prompts or few-shot headers of a serving workload: the input of prefix caching), drawn
    with lengths in prefix_len; the request's own prompt follows the prefix, cut so that the total keeps the drawn length
    when that is longer than the prefix, and at least one own token remains."""
    rng = np.random.default_rng(seed)
    heads = [rng.integers(0, vocab, int(rng.integers(prefix_len[0], prefix_len[1] + 1))).astype(np.int32) for _ in range(n_prefixes)]
    out = []
    for r in reqs:
        r = dict(r)
        if rng.random() < share:
            h = heads[int(rng.integers(0, n_prefixes))]
            own = r["prompt"][: max(1, len(r["prompt"]) - len(h))]
            r["prompt"] = np.concatenate([h, own]).astype(np.int32)
        out.append(r)
    return out


def with_repetition(reqs, vocab, seed, phrase_len=(2, 6), noise=0.0):
    """A copy of the request list whose prompts repeat a short random phrase (2..6 tokens by default), each token replaced
    by a random one with probability `noise`: text that copies from its own context (code edits, summaries, retrieved
    passages), the input on which drafting by lookup in the request's own tokens finds matches. Lengths are kept."""
    rng = np.random.default_rng(seed)
    out = []
    for r in reqs:
        r = dict(r)
        n = len(r["prompt"])
        phrase = rng.integers(0, vocab, int(rng.integers(phrase_len[0], phrase_len[1] + 1)))
        p = np.resize(phrase, n)
        flip = rng.random(n) < noise
        p = np.where(flip, rng.integers(0, vocab, n), p)
        r["prompt"] = p.astype(np.int32)
        out.append(r)
    return out
