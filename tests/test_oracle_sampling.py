"""Pins for the oracle's sampler: brute force on tiny vocabularies, invariants, reductions to
greedy and to plain categorical sampling."""
import numpy as np

from oracle import sampling as S
from oracle.philox import uniform_for_token


def brute_force(logits, T, k, p, u):
    """Independent restatement with explicit Python loops over a fully sorted list."""
    z = [(-(l / T), i) for i, l in enumerate(logits)]
    z.sort()                                   # logit descending, id ascending
    if k and k < len(z):
        z = z[:k]
    m = -z[0][0]
    w = [np.exp(-a - m) for a, _ in z]
    tot = sum(w)
    pr = [x / tot for x in w]
    kept, c = [], 0.0
    for (a, i), q in zip(z, pr):
        kept.append((i, q))
        c += q
        if c >= p:
            break
    tot2 = sum(q for _, q in kept)
    c = 0.0
    for i, q in kept:
        c += q
        if c > u * tot2:
            return i, [i for i, _ in kept]
    return kept[-1][0], [i for i, _ in kept]


def test_matches_brute_force_on_tiny_vocab():
    rng = np.random.default_rng(0)
    for trial in range(600):
        V = int(rng.integers(2, 12))
        logits = rng.standard_normal(V) * 2
        if trial % 3 == 0:
            logits = np.round(logits)          # force ties
        T = float(rng.choice([0.5, 0.8, 1.0, 2.0]))
        k = int(rng.integers(0, V + 2))
        p = float(rng.choice([0.3, 0.9, 1.0]))
        u = float(rng.random())
        d = S.sample_detail(logits, T, k, p, u)
        tok, kept = brute_force(list(logits), T, k, p, u)
        assert d["token"] == tok and list(d["kept"]) == kept


def test_kept_set_invariants():
    rng = np.random.default_rng(1)
    for _ in range(100):
        logits = rng.standard_normal(40)
        d = S.sample_detail(logits, 0.8, 10, 0.9, 0.5)
        top10 = set(np.argsort(-logits)[:10])
        assert set(d["kept"]) <= top10
        pr = d["probs"]
        n = len(d["kept"])
        assert pr[:n].sum() >= 0.9 - 1e-15 or n == 10
        assert n == 1 or pr[: n - 1].sum() < 0.9


def test_greedy_ties_to_lowest_id_and_topk1_is_greedy():
    assert S.greedy([1.0, 3.0, 3.0, 2.0]) == 1
    rng = np.random.default_rng(2)
    for _ in range(50):
        logits = np.round(rng.standard_normal(30) * 2)
        for u in (0.0, 0.5, 0.999):
            assert S.sample_detail(logits, 0.7, 1, 1.0, u)["token"] == S.greedy(logits)


def test_hand_worked_example():
    # probs at T=1: softmax of ln[4,3,2,1] = .4,.3,.2,.1 ; top_k=3 -> .4/.9,.3/.9,.2/.9 ; top_p=.7 keeps two
    logits = np.log([1.0, 4.0, 2.0, 3.0])
    d = S.sample_detail(logits, 1.0, 3, 0.7, 0.0)
    assert list(d["kept"]) == [1, 3]
    assert np.allclose(d["cdf"], [4 / 9, 7 / 9])
    assert S.sample_detail(logits, 1.0, 3, 0.7, 0.5)["token"] == 1      # 0.5 * 7/9 = .389 < .444
    assert S.sample_detail(logits, 1.0, 3, 0.7, 0.6)["token"] == 3      # .467 > .444
    # temperature divides the logits: T=.5 squares the odds -> 16,9,4,1
    d = S.sample_detail(logits, 0.5, 0, 1.0, 0.0)
    assert np.allclose(d["probs"], np.array([16, 9, 4, 1]) / 30.0)


def test_plain_categorical_frequencies():
    logits = np.log([0.5, 0.25, 0.125, 0.125])
    n = 8000
    cnt = np.zeros(4)
    for i in range(n):
        cnt[S.sample(logits, 1.0, 0, 1.0, 99, i)] += 1
    exp = n * np.array([0.5, 0.25, 0.125, 0.125])
    assert ((cnt - exp) ** 2 / exp).sum() < 21.0   # 3 dof, p ~ 1e-4


def test_draw_uses_the_output_index_as_counter():
    logits = np.zeros(16)
    for i in (0, 5):
        u = uniform_for_token(1234, i)
        assert S.sample(logits, 1.0, 0, 1.0, 1234, i) == int(u * 16)


def test_decision_guard_of_the_gpu_tests_is_sound():
    """tests/parity.sampling_decisions_clear says when a sampled token may be compared exactly although the engine's
    logits differ from the oracle's by up to tol: whenever it says "clear", the oracle's sampler on logits perturbed by
    any error within tol must return the same token. For the other tokens the GPU tests require
    sampled_token_plausible: it must accept every token the sampler returns on perturbed logits (no false alarms) and
    reject most wrong tokens. Checked with random and with adversarial (sign-pattern) errors."""
    from tests.parity import sampling_decisions_clear, sampled_token_plausible
    from oracle.philox import uniform_for_token
    rng = np.random.default_rng(11)
    clear = wrong = wrong_rejected = 0
    for trial in range(600):
        V = int(rng.choice([60, 400, 2500]))
        row = rng.normal(0.0, float(rng.choice([0.4, 1.3])), V)
        r = dict(temperature=float(rng.choice([0.3, 0.8, 1.0])), top_k=int(rng.choice([5, 50, 0 if V <= 400 else 40])),
                 top_p=float(rng.choice([0.5, 0.9, 1.0])), seed=int(rng.integers(1, 1 << 40)))
        u = uniform_for_token(r["seed"], trial)
        d = S.sample_detail(row, r["temperature"], r["top_k"], r["top_p"], u)
        tol = float(rng.choice([1e-3, 5e-3, 2e-2])) * np.abs(row).max()
        is_clear = sampling_decisions_clear(row, r, d, tol)
        clear += int(is_clear)
        order = S.candidate_order(row)
        pos = int(np.nonzero(order == d["token"])[0][0])
        for rep in range(12):
            if rep < 6:
                e = rng.uniform(-tol, tol, V)
            else:                      # worst cases: everything ahead of the chosen token pushed one way, the rest the other
                e = np.full(V, tol if rep % 2 else -tol)
                e[order[:pos + (rep % 3 == 0)]] *= -1.0
            g = S.sample_detail(row + e, r["temperature"], r["top_k"], r["top_p"], u)["token"]
            if is_clear:
                assert g == d["token"], (trial, rep)
            assert sampled_token_plausible(row, r, d, g, tol), (trial, rep, g, d["token"])
        # a token from elsewhere in the distribution (what a wrong uniform, seed or counter would give) is mostly rejected
        other = S.sample_detail(row, r["temperature"], r["top_k"], r["top_p"], float(rng.random()))["token"]
        if other != d["token"] and tol <= 5e-3 * np.abs(row).max():
            wrong += 1
            wrong_rejected += int(not sampled_token_plausible(row, r, d, other, tol))
    assert clear > 60
    assert wrong > 100 and wrong_rejected > 0.7 * wrong, (wrong, wrong_rejected)
