"""The sampler kernel on its own (blink_sample_rows: logits in, tokens out through the C ABI) against the oracle's
sampler on crafted rows: every stage of the top-k selection (one-pass per-thread top-4, counting search, radix select
on massive ties), top_k from 1 to 1024 and 0, greedy ties, and rows of the benchmark's vocabulary size.

The engine orders candidates by the exact fp32 logits (ties to the lower id), as the oracle does on the same values
widened to fp64, so top-k membership and order are compared without a tolerance. Its exponentials and cumulative sums
are fp32 (sums of up to 1024 terms): a row whose top-p cut or CDF bin lies within 2e-5 of a boundary is counted as
undecided instead (and at least 80 % of the rows of every test must be decided; the tie cases all are)."""
import numpy as np
import pytest

from oracle import sampling as S
from oracle.philox import uniform_for_token

pytestmark = pytest.mark.gpu

from tests.parity import arithmetic_decided as decided


def check(lib, rows, params, token_index, min_decided=0.8):
    rows = np.ascontiguousarray(rows, dtype=np.float32)
    got = lib.sample_rows(rows, params, token_index)
    n_dec = 0
    for r in range(rows.shape[0]):
        p, row = params[r], rows[r].astype(np.float64)
        if p["temperature"] == 0.0:
            assert int(got[r]) == S.greedy(row), (r, int(got[r]), S.greedy(row))
            n_dec += 1
            continue
        d = S.sample_detail(row, p["temperature"], p["top_k"], p["top_p"], uniform_for_token(p["seed"], int(token_index[r])))
        if decided(d, p["top_p"]):
            assert int(got[r]) == d["token"], (r, int(got[r]), d["token"], p)
            n_dec += 1
        else:
            assert int(got[r]) in set(int(x) for x in d["kept"]) | set(int(x) for x in S.candidate_order(row)[: len(d["kept"]) + 1])
    assert n_dec >= min_decided * rows.shape[0], (n_dec, rows.shape[0])
    return n_dec


def P(temperature=0.8, top_k=50, top_p=0.9, seed=1):
    return dict(temperature=temperature, top_k=top_k, top_p=top_p, seed=seed)


def test_random_rows_small_vocab_every_top_k(lib):
    rng = np.random.default_rng(1)
    V = 5000
    ks = [1, 2, 4, 5, 40, 50, 255, 256, 257, 300, 511, 1000, 1024]
    rows = rng.normal(0.0, 1.3, (len(ks) * 4, V))
    params = [P(top_k=ks[i % len(ks)], top_p=[0.9, 1.0, 0.5, 0.97][i // len(ks)], seed=1000 + i) for i in range(rows.shape[0])]
    n = check(lib, rows, params, np.arange(rows.shape[0]) % 7)
    print("decided", n, "of", rows.shape[0])


def test_top_k_zero_and_beyond_the_vocabulary(lib):
    rng = np.random.default_rng(2)
    for V in (1000, 1024, 37):            # top_k = 0 keeps the whole vocabulary (allowed up to 1024 entries); 37: unaligned rows
        rows = rng.normal(0.0, 2.0, (6, V))
        params = [P(top_k=0, top_p=1.0, temperature=1.0, seed=5 + i) for i in range(3)] + [P(top_k=V + 100, top_p=0.8, seed=9 + i) for i in range(3)]
        check(lib, rows, params, np.arange(6))


def test_more_than_four_of_the_top_k_in_one_threads_stripe(lib):
    """The one-pass stage keeps four keys per thread; thread 0 visits ids 0-3, 1024-1027, 2048-..: with seven of the
    largest logits there it drops keys above the threshold and the counting search takes over."""
    rng = np.random.default_rng(3)
    V = 8192
    rows = rng.normal(0.0, 1.0, (8, V))
    hot = [0, 1, 2, 3, 1024, 1025, 2048, 4097, 6000]
    for r in range(rows.shape[0]):
        rows[r, hot] = 6.0 + rng.random(len(hot))
    params = [P(top_k=[50, 20, 9, 256][r % 4], top_p=0.93, seed=77 + r) for r in range(rows.shape[0])]
    check(lib, rows, params, np.arange(rows.shape[0]) + 3)


def test_massive_ties_take_the_radix_select(lib):
    """All logits equal, or thousands tied at the maximum: the counting search finds no threshold that keeps at most 1024
    keys, and the exact radix select on (logit, id) decides; the kept candidates are the lowest ids."""
    V = 8192
    flat = np.full((4, V), 0.25)
    params = [P(top_k=300, top_p=0.915, seed=11), P(top_k=1024, top_p=0.3335, seed=12), P(top_k=257, top_p=1.0, seed=13),
              P(top_k=50, top_p=0.91, seed=14)]
    check(lib, flat, params, [0, 1, 2, 3], min_decided=1.0)
    # ties at the maximum placed so that thread 0's stripe (ids 0-3 mod 1024) holds more than four of the lowest tied ids
    rng = np.random.default_rng(4)
    rows = rng.normal(0.0, 1.0, (3, V))
    tied = sorted(set([j * 1024 + i for j in range(8) for i in range(4)]) | set(int(x) for x in rng.choice(np.arange(5000, V), 2000, replace=False)))
    rows[:, tied] = 7.5
    params = [P(top_k=50, top_p=0.91, seed=21), P(top_k=20, top_p=0.77, seed=22), P(top_k=256, top_p=0.99, seed=23)]
    check(lib, rows, params, [5, 6, 7], min_decided=1.0)
    # greedy on ties: the lowest id
    g = np.zeros((2, 3001))
    g[0, [17, 2900, 18]] = 1.0
    g[1, :] = -3.0
    check(lib, g, [P(temperature=0.0), P(temperature=0.0)], [0, 0], min_decided=1.0)


def test_rows_of_the_benchmark_vocabulary(lib):
    """V = 128256, top-k 50 / top-p 0.9 / T 0.8 as the llama3_8b workload samples, logits spread like that model's."""
    rng = np.random.default_rng(5)
    V = 128256
    rows = rng.normal(0.0, 1.28, (24, V)).astype(np.float32)
    params = [P(seed=int(rng.integers(1, 1 << 62))) for _ in range(16)] + [P(temperature=0.0)] * 4 + [P(top_k=1024, top_p=0.95, seed=3)] * 4
    n = check(lib, rows, params, rng.integers(0, 1000, 24))
    print("decided", n, "of 24")


def test_parameter_errors(lib):
    rows = np.zeros((1, 2000), dtype=np.float32)
    for bad in (P(top_k=0), P(top_k=2000), P(top_p=0.0), P(temperature=-1.0)):
        with pytest.raises(lib.BlinkError) as ei:
            lib.sample_rows(rows, [bad], [0])
        assert ei.value.code == lib.ERR_INVAL
