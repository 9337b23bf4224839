"""Pins for the oracle's transformer: closed forms, special cases, an independent stock-torch
implementation, and agreement of the dense / cached / paged variants."""
import numpy as np
import pytest
import torch

import synth
from oracle import model as M

CFG = dict(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=50, dtype=0,
           rms_eps=1e-5, rope_theta=10000.0)


def weights(cfg=CFG, seed=7, std=0.3, jitter=0.2):
    raw = synth.make_weights(cfg, seed, std=std, gain_jitter=jitter)
    return raw, M.Weights(cfg, raw)


def test_rmsnorm_unit_rms_and_gain():
    x = np.random.default_rng(0).standard_normal((5, 64)) * 3
    y = M.rmsnorm(x, np.ones(64), 0.0)
    assert np.allclose(np.sqrt((y * y).mean(-1)), 1.0, atol=1e-12)
    g = np.linspace(0.5, 2, 64)
    assert np.allclose(M.rmsnorm(x, g, 0.0), y * g)
    # eps sits inside the square root, added to the mean square
    z = M.rmsnorm(np.full((1, 4), 2.0), np.ones(4), 5.0)
    assert np.allclose(z, 2.0 / 3.0)


def test_rope_identity_norm_relative_and_pairing():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((6, 3, 16))
    assert np.allclose(M.rope(x, np.zeros(6), 1e4), x)
    y = M.rope(x, np.arange(6) * 7, 1e4)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1))
    q, k = rng.standard_normal((1, 1, 16)), rng.standard_normal((1, 1, 16))
    d1 = (M.rope(q, [9], 1e4) * M.rope(k, [4], 1e4)).sum()
    d2 = (M.rope(q, [105], 1e4) * M.rope(k, [100], 1e4)).sum()
    assert abs(d1 - d2) < 1e-9
    # pairing i <-> i + hd/2, angle pos * theta^(-2i/hd): one-hot input, hand-computed
    e = np.zeros((1, 1, 16)); e[0, 0, 3] = 1.0
    r = M.rope(e, [2], 100.0)[0, 0]
    ang = 2 * 100.0 ** (-2 * 3 / 16)
    exp = np.zeros(16); exp[3] = np.cos(ang); exp[11] = np.sin(ang)
    assert np.allclose(r, exp)


def test_prompt_of_one_attends_to_itself_only():
    raw, W = weights()
    cfg = CFG
    x = W["embed"][[5]]
    q, k, v = M._qkv(cfg, W, 0, x, np.array([0]))
    out = M._attend(cfg, q[0], k, v)
    for h in range(4):
        assert np.allclose(out[h], v[0, h // 2])


def test_equal_keys_give_mean_of_values():
    rng = np.random.default_rng(2)
    K = np.repeat(rng.standard_normal((1, 2, 16)), 7, axis=0)
    V = rng.standard_normal((7, 2, 16))
    q = rng.standard_normal((4, 16))
    out = M._attend(CFG, q, K, V)
    for h in range(4):
        assert np.allclose(out[h], V[:, h // 2].mean(0))


def test_attention_scale_is_inverse_sqrt_head_dim():
    # two keys, scores differ by exactly ln(3)*sqrt(hd) before scaling -> weights 3:1
    hd = 16
    cfg = dict(CFG, n_q_heads=1, n_kv_heads=1)
    q = np.zeros((1, hd)); q[0, 0] = 1.0
    K = np.zeros((2, 1, hd)); K[0, 0, 0] = np.log(3.0) * np.sqrt(hd)
    V = np.zeros((2, 1, hd)); V[0, 0, 0] = 1.0; V[1, 0, 1] = 1.0
    out = M._attend(cfg, q, K, V)[0]
    assert np.allclose(out[:2], [0.75, 0.25])


def test_zero_output_projections_reduce_to_one_gemv():
    raw, _ = weights()
    raw = dict(raw)
    for l in range(2):
        raw[f"l{l}.wo"] = np.zeros_like(raw[f"l{l}.wo"])
        raw[f"l{l}.wd"] = np.zeros_like(raw[f"l{l}.wd"])
    W = M.Weights(CFG, raw)
    toks = [3, 9, 11]
    got = M.forward_dense(CFG, W, toks)
    e = raw["embed"].astype(np.float64)[toks]
    h = e / np.sqrt((e * e).mean(-1, keepdims=True) + 1e-5) * raw["gf"].astype(np.float64)
    assert np.allclose(got, h @ raw["lm"].astype(np.float64).T, atol=1e-13)


def torch_reference(cfg, raw, tokens):
    """The same architecture with stock torch CPU ops, written independently: complex-number rotary,
    scaled_dot_product_attention, repeat_interleave for grouped heads."""
    f = lambda n: torch.from_numpy(np.asarray(raw[n], dtype=np.float64) if raw[n].dtype != np.uint16
                                   else synth.bf16_bits_to_f32(raw[n]).astype(np.float64))
    nq, nkv, hd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    T = len(tokens)
    x = f("embed")[torch.tensor(tokens)]
    freqs = torch.outer(torch.arange(T, dtype=torch.float64),
                        cfg["rope_theta"] ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd))
    rot = torch.polar(torch.ones_like(freqs), freqs)  # e^{i pos w_j}

    def rotary(t):  # [T, H, hd], first half = real parts, second half = imaginary parts
        z = torch.complex(t[..., : hd // 2], t[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], -1)

    def norm(t, g):
        return t * torch.rsqrt(t.pow(2).mean(-1, keepdim=True) + cfg["rms_eps"]) * g

    for l in range(cfg["n_layers"]):
        h = norm(x, f(f"l{l}.g1"))
        q = rotary(torch.nn.functional.linear(h, f(f"l{l}.wq")).view(T, nq, hd))
        k = rotary(torch.nn.functional.linear(h, f(f"l{l}.wk")).view(T, nkv, hd))
        v = torch.nn.functional.linear(h, f(f"l{l}.wv")).view(T, nkv, hd)
        k = k.repeat_interleave(nq // nkv, dim=1)
        v = v.repeat_interleave(nq // nkv, dim=1)
        a = torch.nn.functional.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1),
                                                             is_causal=True)
        x = x + torch.nn.functional.linear(a.transpose(0, 1).reshape(T, nq * hd), f(f"l{l}.wo"))
        h = norm(x, f(f"l{l}.g2"))
        x = x + torch.nn.functional.linear(
            torch.nn.functional.silu(torch.nn.functional.linear(h, f(f"l{l}.wg"))) * torch.nn.functional.linear(h, f(f"l{l}.wu")),
            f(f"l{l}.wd"))
    return torch.nn.functional.linear(norm(x, f("gf")), f("lm")).numpy()


@pytest.mark.parametrize("cfg", [CFG, dict(CFG, n_kv_heads=4), dict(CFG, n_kv_heads=1, dtype=1)])
def test_matches_stock_torch_implementation(cfg):
    raw, W = weights(cfg)
    toks = list(np.random.default_rng(3).integers(0, cfg["vocab"], 13))
    ref = torch_reference(cfg, raw, toks)
    got = M.forward_dense(cfg, W, toks)
    assert np.abs(got - ref).max() < 1e-10 * max(1.0, np.abs(ref).max())


def test_dense_cached_and_paged_variants_agree():
    raw, W = weights()
    rng = np.random.default_rng(4)
    toks = list(rng.integers(0, 50, 21))
    dense = M.forward_dense(CFG, W, toks)
    m = M.CachedModel(CFG, W)
    l0 = m.step(toks[:9])
    assert np.abs(l0 - dense[8]).max() < 1e-12
    for i in range(9, 21):
        li = m.step([toks[i]])
        assert np.abs(li - dense[i]).max() < 1e-12
    # paged: two sequences interleaved in one pool with a scrambled block order, block size 4
    bs = 4
    kv = M.PagedKV(CFG, 16, bs)
    perm = list(rng.permutation(16))
    bt = [perm[:6], perm[6:12]]
    seqs = [toks, list(rng.integers(0, 50, 17))]
    dense2 = M.forward_dense(CFG, W, seqs[1])
    P = [9, 5]
    ids, pos, slot, ts, last = [], [], [], [], []
    for s in range(2):
        for p in range(P[s]):
            ids.append(seqs[s][p]); pos.append(p); slot.append(bt[s][p // bs] * bs + p % bs); ts.append(s)
        last.append(len(ids) - 1)
    lg = M.paged_forward(CFG, W, kv, ids, pos, slot, ts, bt, last)
    assert np.abs(lg[0] - dense[8]).max() < 1e-12 and np.abs(lg[1] - dense2[4]).max() < 1e-12
    for step in range(8):
        ids = [seqs[s][P[s] + step] for s in range(2)]
        pos = [P[s] + step for s in range(2)]
        slot = [bt[s][p // bs] * bs + p % bs for s, p in enumerate(pos)]
        lg = M.paged_forward(CFG, W, kv, ids, pos, slot, [0, 1], bt, [0, 1])
        assert np.abs(lg[0] - dense[pos[0]]).max() < 1e-12
        assert np.abs(lg[1] - dense2[pos[1]]).max() < 1e-12


def test_bruteforce_generation_equals_cached_generation():
    from oracle import serve as SV
    raw, W = weights()
    req = dict(prompt=np.array([1, 2, 3, 4, 5]), max_new_tokens=6, temperature=0.0, top_k=0, top_p=1.0, seed=1)
    a = SV.generate_reference(CFG, W, req)
    b = M.generate_bruteforce(CFG, W, req["prompt"], 6, lambda lg, i: int(np.argmax(lg)))
    assert a == b


# ---- mixture of experts ------------------------------------------------------------------------------------------------

def _moe_cfg(E=6, k=2):
    return dict(synth.model_config("tiny"), n_layers=2, vocab=61, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=24,
                n_experts=E, n_active=k)


def test_moe_with_one_expert_is_the_dense_model():
    """One expert, one active: the router's weight is softmax over a single logit = 1, so the layer is the plain FFN with
    that expert's matrices (the dense model is pinned above)."""
    cfg = _moe_cfg(1, 1)
    raw = synth.make_weights(cfg, 3, gain_jitter=0.1)
    dense_cfg = dict(cfg, n_experts=0, n_active=0)
    dense_raw = {k: (v[0] if k.endswith((".wg", ".wu", ".wd")) else v) for k, v in raw.items() if not k.endswith(".wr")}
    toks = np.arange(11) % 61
    a = M.forward_dense(cfg, M.Weights(cfg, raw), toks)
    b = M.forward_dense(dense_cfg, M.Weights(dense_cfg, dense_raw), toks)
    assert np.abs(a - b).max() < 1e-12


def test_moe_all_experts_active_with_a_zero_router_is_the_mean_of_the_experts():
    cfg = _moe_cfg(4, 4)
    raw = synth.make_weights(cfg, 4)
    for l in range(2):
        raw[f"l{l}.wr"] = np.zeros_like(raw[f"l{l}.wr"])
    W = M.Weights(cfg, raw)
    h = np.random.default_rng(0).normal(size=(5, 32))
    got = M.moe_ffn(cfg, W, 0, h)
    want = np.mean([(M.silu(h @ W["l0.wg"][e].T) * (h @ W["l0.wu"][e].T)) @ W["l0.wd"][e].T for e in range(4)], axis=0)
    assert np.abs(got - want).max() < 1e-12


def test_moe_routing_by_hand_ties_and_forced_selection():
    """Router logits written by hand: the two largest win, a tie goes to the lower expert id, the weights are the softmax
    over the two selected logits (1 : e^-1 here); forcing another selection changes the output accordingly; relabelling
    the experts does not change the layer."""
    cfg = _moe_cfg(5, 2)
    sel, margin = M.route(cfg, np.array([0.5, 2.0, 1.0, 2.0, 1.0]))
    assert list(sel) == [1, 3] and margin == 1.0
    sel, margin = M.route(cfg, np.array([1.0, 0.0, 1.0, 1.0, -1.0]))
    assert list(sel) == [0, 2] and margin == 0.0
    raw = synth.make_weights(cfg, 5)
    W = M.Weights(cfg, raw)
    rng = np.random.default_rng(1)
    h = rng.normal(size=(1, 32))
    wr = np.zeros((5, 32))
    wr[1] = 2.0 * h[0] / (h[0] @ h[0])          # logit 2 for expert 1
    wr[4] = 1.0 * h[0] / (h[0] @ h[0])          # logit 1 for expert 4, 0 for the rest
    W._cache["l0.wr"] = wr
    f = lambda e: (M.silu(W["l0.wg"][e] @ h[0]) * (W["l0.wu"][e] @ h[0])) @ W["l0.wd"][e].T
    w1, w4 = 1.0 / (1.0 + np.exp(-1.0)), np.exp(-1.0) / (1.0 + np.exp(-1.0))
    log = []
    assert np.abs(M.moe_ffn(cfg, W, 0, h, route_log=log)[0] - (w1 * f(1) + w4 * f(4))).max() < 1e-12
    assert list(log[0]["own"][0]) == [1, 4] and abs(log[0]["margin"][0] - 1.0) < 1e-12
    forced = M.moe_ffn(cfg, W, 0, h, routing=[[1, 0]])[0]       # expert 0 has logit 0: weights 1 : e^-2
    assert np.abs(forced - (f(1) + np.exp(-2.0) * f(0)) / (1.0 + np.exp(-2.0))).max() < 1e-12
    perm = np.array([3, 0, 4, 1, 2])
    for n in ("wg", "wu", "wd"):
        W._cache[f"l1.{n}"] = W[f"l0.{n}"][perm]
    W._cache["l1.wr"] = wr[perm]
    assert np.abs(M.moe_ffn(cfg, W, 1, h) - M.moe_ffn(cfg, W, 0, h)).max() < 1e-12


def test_moe_dense_equals_cached_equals_paged():
    cfg = _moe_cfg()
    raw = synth.make_weights(cfg, 6, gain_jitter=0.1)
    W = M.Weights(cfg, raw)
    toks = np.random.default_rng(2).integers(0, 61, 23)
    dense = M.forward_dense(cfg, W, toks)
    m = M.CachedModel(cfg, W)
    got = [m.step(toks[:9])] + [m.step([t]) for t in toks[9:]]
    assert np.abs(np.array(got) - dense[8:]).max() < 1e-12
    kv = M.PagedKV(cfg, 4, 8)
    bt = [[2, 0, 3]]
    lg = M.paged_forward(cfg, W, kv, list(toks), list(range(23)), [bt[0][p // 8] * 8 + p % 8 for p in range(23)], [0] * 23, bt, [22])
    assert np.abs(lg[0] - dense[22]).max() < 1e-12


def test_routing_check_accepts_the_own_routing_and_rejects_planted_mistakes():
    """tests/parity.check_routing (used by the GPU tests of the expert selection): the oracle's own routing passes; a
    clearly rejected expert in place of a selected one, two clearly ordered experts swapped, or one expert twice, fail.
    The report's `gaps` is the smallest difference between consecutive selected logits."""
    from tests.parity import check_routing, ROUTE_MARGIN
    cfg = _moe_cfg(6, 3)
    raw = synth.make_weights(cfg, 8, std=0.3)
    W = M.Weights(cfg, raw)
    h = np.random.default_rng(3).normal(size=(40, 32))
    logs = []
    for l in range(2):
        M.moe_ffn(cfg, W, l, h, route_log=logs)
    own = np.stack([lg["own"] for lg in logs])
    r = h @ W["l0.wr"].T
    picked = np.take_along_axis(r, logs[0]["own"], axis=1)
    assert np.allclose(logs[0]["gaps"], np.minimum(picked[:, 0] - picked[:, 1], picked[:, 1] - picked[:, 2]))
    stats = dict(pairs=0, unclear=0)
    check_routing(cfg, own, logs, stats)
    assert stats["pairs"] == 80
    t = int(np.argmax(np.minimum(logs[0]["margin"], logs[0]["gaps"]) / logs[0]["scale"]))     # the clearest token of layer 0
    assert min(logs[0]["margin"][t], logs[0]["gaps"][t]) > ROUTE_MARGIN * logs[0]["scale"][t]
    rejected = [e for e in range(6) if e not in own[0, t]][0]
    for wrong in ([own[0, t, 0], own[0, t, 1], rejected], [own[0, t, 1], own[0, t, 0], own[0, t, 2]], [own[0, t, 0]] * 3):
        bad = own.copy()
        bad[0, t] = wrong
        with pytest.raises(AssertionError):
            check_routing(cfg, bad, logs, dict(pairs=0, unclear=0))
