"""Seeded random weights and the flat blob format handed to the engine.

Every matrix is stored row-major as [out_features][in_features]. Order of tensors in the
blob (see tensor_order): embed [V][d]; per layer g1 [d], wq [nq*hd][d], wk [nkv*hd][d],
wv [nkv*hd][d], wo [d][nq*hd], g2 [d], wg [F][d], wu [F][d], wd [d][F]; then gf [d],
lm [V][d]. A mixture-of-experts model (n_experts = E > 0, d_ffn = width of one expert) has per layer, in place of
wg, wu, wd: the router wr [E][d], then wg [E][F][d], wu [E][F][d], wd [E][d][F]. Norm gains (g1, g2, gf) are always fp32. Matrices are fp32 (dtype 0) or bf16
bit patterns (dtype 1, uint16, produced by round-to-nearest-even of the fp32 draw): those
bits are the weights for every consumer.
"""
import numpy as np
from concurrent.futures import ThreadPoolExecutor


def f32_to_bf16_bits(a):
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16). Inputs are finite."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def tensor_order(cfg):
    """[(name, shape, is_gain)] in blob order."""
    d, hd = cfg["d_model"], cfg["head_dim"]
    nq, nkv, F, V = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["d_ffn"], cfg["vocab"]
    E = cfg.get("n_experts", 0)
    out = [("embed", (V, d), False)]
    for l in range(cfg["n_layers"]):
        out += [(f"l{l}.g1", (d,), True), (f"l{l}.wq", (nq * hd, d), False), (f"l{l}.wk", (nkv * hd, d), False),
                (f"l{l}.wv", (nkv * hd, d), False), (f"l{l}.wo", (d, nq * hd), False), (f"l{l}.g2", (d,), True)]
        if E:   # mixture of experts: router, then the experts' matrices stacked
            out += [(f"l{l}.wr", (E, d), False), (f"l{l}.wg", (E, F, d), False), (f"l{l}.wu", (E, F, d), False), (f"l{l}.wd", (E, d, F), False)]
        else:
            out += [(f"l{l}.wg", (F, d), False), (f"l{l}.wu", (F, d), False), (f"l{l}.wd", (d, F), False)]
    out += [("gf", (d,), True), ("lm", (V, d), False)]
    return out


def make_weights(cfg, seed, std=0.02, gain_jitter=0.0, threads=8):
    """dict name -> ndarray. Matrices ~ N(0, std) (fp32, or bf16 bits as uint16 when dtype == 1);
    gains are 1 (+ gain_jitter * N(0,1), test-only) in fp32. Each tensor has its own child seed, so
    the result does not depend on the thread count."""
    order = tensor_order(cfg)
    children = np.random.SeedSequence(seed).spawn(len(order))

    def one(i):
        name, shape, is_gain = order[i]
        rng = np.random.default_rng(children[i])
        if is_gain:
            g = np.ones(shape, dtype=np.float32)
            if gain_jitter:
                g = (g + gain_jitter * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)
            return name, g
        n = int(np.prod(shape))
        flat = np.empty(n, dtype=np.uint16 if cfg["dtype"] == 1 else np.float32)
        step = 1 << 24
        for s in range(0, n, step):
            w = rng.standard_normal(min(step, n - s), dtype=np.float32) * np.float32(std)
            flat[s:s + len(w)] = f32_to_bf16_bits(w) if cfg["dtype"] == 1 else w
        return name, flat.reshape(shape)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        return dict(ex.map(one, range(len(order))))


def pack_blob(cfg, weights):
    """Concatenate the tensors in blob order into one contiguous uint8 array."""
    parts = [np.ascontiguousarray(weights[name]).reshape(-1).view(np.uint8) for name, _, _ in tensor_order(cfg)]
    total = sum(p.size for p in parts)
    blob = np.empty(total, dtype=np.uint8)
    o = 0
    for p in parts:
        blob[o:o + p.size] = p
        o += p.size
    return blob
