"""Decoder-only transformer of the serving step, fp64. Oracle code: test infrastructure only.

The paper treats the model as an opaque engine (section 4.3); the workloads fix a
Llama-style decoder: token embedding, per layer RMSNorm -> Q/K/V projections -> rotary
embedding (rotate-half pairing) -> causal attention with grouped KV heads -> output
projection + residual -> RMSNorm -> SiLU-gated FFN + residual; final RMSNorm and an untied
LM head. No biases. All arithmetic is fp64 on the stored weight values, with no rounding of
activations or cached K/V.

Mixture-of-experts variant (n_experts > 0; the second workload of the paper's evaluation, section 6, is such a model
and the paper fixes nothing about it either): the FFN of every layer is replaced by n_experts SiLU-gated FFNs of width
d_ffn and a router matrix [n_experts][d]. Per token: router logits r = h Wr^T; the n_active largest are selected (ties to
the lower expert id); their weights are the softmax over the selected logits (softmax over all experts, then
renormalised over the selected ones, is the same thing); the layer adds sum_j w_j FFN_{e_j}(h). The selection is an
integer decision taken from floating-point values: a caller may force it (`routing`) and receives the oracle's own choice
and its margin (`route_log`), so that a test can require agreement wherever the margin exceeds the tolerance.

Three variants compute the same function:
  forward_dense: the definition. All positions at once, dense causal attention, no cache.
  CachedModel:   contiguous per-sequence KV cache, prefill then one token at a time.
  paged_forward: K/V live in a block pool addressed through block tables and a slot
                 mapping, many sequences per call (what the serving loop uses).
"""
import numpy as np

from synth.weights import bf16_bits_to_f32


class Weights:
    """fp64 view of a weight dict from synth.make_weights (bf16 bits are widened exactly)."""

    def __init__(self, cfg, raw, cache=True):
        self.cfg = cfg
        self.raw = raw
        self._cache = {} if cache else None

    def __getitem__(self, name):
        if self._cache is not None and name in self._cache:
            return self._cache[name]
        a = self.raw[name]
        if a.dtype == np.uint16:
            a = bf16_bits_to_f32(a)
        a = a.astype(np.float64)
        if self._cache is not None:
            self._cache[name] = a
        return a


def rmsnorm(x, g, eps):
    return x * g / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)


def rope(x, pos, theta):
    """x: [T, H, hd], pos: [T]. Pairs dimension i with i + hd/2; angle pos * theta**(-2i/hd)."""
    hd = x.shape[-1]
    half = hd // 2
    inv = theta ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z):
    return z / (1.0 + np.exp(-z))


def _qkv(cfg, W, l, x, pos):
    nq, nkv, hd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    h = rmsnorm(x, W[f"l{l}.g1"], cfg["rms_eps"])
    T = x.shape[0]
    q = (h @ W[f"l{l}.wq"].T).reshape(T, nq, hd)
    k = (h @ W[f"l{l}.wk"].T).reshape(T, nkv, hd)
    v = (h @ W[f"l{l}.wv"].T).reshape(T, nkv, hd)
    return rope(q, pos, cfg["rope_theta"]), rope(k, pos, cfg["rope_theta"]), v


def _attend(cfg, q, K, V):
    """q: [nq, hd] at the last of the positions held in K, V: [n, nkv, hd]. Softmax over all n."""
    nq, nkv, hd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    out = np.empty((nq, hd))
    for h in range(nq):
        kvh = h // (nq // nkv)
        s = K[:, kvh, :] @ q[h] / np.sqrt(hd)
        p = np.exp(s - s.max())
        p /= p.sum()
        out[h] = p @ V[:, kvh, :]
    return out


def route(cfg, r):
    """r: router logits [E] of one token. Returns (selected expert ids in order of decreasing logit, ties to the lower
    id; margin between the last selected and the first rejected logit, inf when all experts are selected)."""
    E, k = cfg["n_experts"], cfg["n_active"]
    order = np.lexsort((np.arange(E), -r))
    margin = float(r[order[k - 1]] - r[order[k]]) if k < E else np.inf
    return order[:k], margin


def moe_ffn(cfg, W, l, h, routing=None, route_log=None):
    """h: normalised input [T][d]. routing: optional [T][n_active] expert ids to use instead of the own selection."""
    T = h.shape[0]
    r = h @ W[f"l{l}.wr"].T
    out = np.zeros_like(h)
    own, margins = [], []
    for t in range(T):
        sel, margin = route(cfg, r[t])
        own.append(sel)
        margins.append(margin)
        if routing is not None:
            sel = np.asarray(routing[t], dtype=np.int64)
        w = np.exp(r[t, sel] - r[t, sel].max())
        w /= w.sum()
        for wj, e in zip(w, sel):
            out[t] += wj * ((silu(W[f"l{l}.wg"][e] @ h[t]) * (W[f"l{l}.wu"][e] @ h[t])) @ W[f"l{l}.wd"][e].T)
    if route_log is not None:
        own = np.array(own)
        picked = np.take_along_axis(r, own, axis=1)     # the selected logits, in selection order
        gaps = (picked[:, :-1] - picked[:, 1:]).min(axis=1) if own.shape[1] > 1 else np.full(T, np.inf)
        route_log.append(dict(layer=l, own=own, margin=np.array(margins), gaps=gaps, scale=np.abs(r).max(axis=1)))
    return out


def _post_attention(cfg, W, l, x, attn, routing=None, route_log=None):
    T = x.shape[0]
    x = x + attn.reshape(T, -1) @ W[f"l{l}.wo"].T
    h = rmsnorm(x, W[f"l{l}.g2"], cfg["rms_eps"])
    if cfg.get("n_experts", 0):
        return x + moe_ffn(cfg, W, l, h, None if routing is None else routing[l], route_log)
    return x + (silu(h @ W[f"l{l}.wg"].T) * (h @ W[f"l{l}.wu"].T)) @ W[f"l{l}.wd"].T


def _head(cfg, W, x):
    return rmsnorm(x, W["gf"], cfg["rms_eps"]) @ W["lm"].T


def forward_dense(cfg, W, tokens, all_positions=True):
    """Logits [T][V] (or [V] of the last position) of one sequence by the plain definition:
    full score matrix per head, causal mask, row softmax."""
    tokens = np.asarray(tokens)
    T = tokens.size
    nq, nkv, hd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    pos = np.arange(T)
    future = pos[None, :] > pos[:, None]
    x = W["embed"][tokens]
    for l in range(cfg["n_layers"]):
        q, k, v = _qkv(cfg, W, l, x, pos)
        attn = np.empty_like(q)
        for h in range(nq):
            kvh = h // (nq // nkv)
            s = q[:, h, :] @ k[:, kvh, :].T / np.sqrt(hd)
            s[future] = -np.inf
            p = np.exp(s - s.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            attn[:, h, :] = p @ v[:, kvh, :]
        x = _post_attention(cfg, W, l, x, attn)
    return _head(cfg, W, x) if all_positions else _head(cfg, W, x[-1:])[0]


class CachedModel:
    """One sequence with a contiguous KV cache."""

    def __init__(self, cfg, W):
        self.cfg, self.W = cfg, W
        self.K = [np.zeros((0, cfg["n_kv_heads"], cfg["head_dim"])) for _ in range(cfg["n_layers"])]
        self.V = [np.zeros((0, cfg["n_kv_heads"], cfg["head_dim"])) for _ in range(cfg["n_layers"])]
        self.n = 0

    def step(self, tokens):
        """Append tokens (a prompt, or one decode token); return the logits of the last one."""
        cfg, W = self.cfg, self.W
        tokens = np.atleast_1d(np.asarray(tokens))
        T = tokens.size
        pos = self.n + np.arange(T)
        x = W["embed"][tokens]
        for l in range(cfg["n_layers"]):
            q, k, v = _qkv(cfg, W, l, x, pos)
            self.K[l] = np.concatenate([self.K[l], k])
            self.V[l] = np.concatenate([self.V[l], v])
            attn = np.empty_like(q)
            for t in range(T):
                n = self.n + t + 1
                attn[t] = _attend(cfg, q[t], self.K[l][:n], self.V[l][:n])
            x = _post_attention(cfg, W, l, x, attn)
        self.n += T
        return _head(cfg, W, x[-1:])[0]


class PagedKV:
    """Block pool: K and V as [layer][n_blocks*block_size][nkv][hd], addressed by slot = block*bs + offset."""

    def __init__(self, cfg, n_blocks, bs):
        shape = (cfg["n_layers"], n_blocks * bs, cfg["n_kv_heads"], cfg["head_dim"])
        self.K = np.full(shape, np.nan)
        self.V = np.full(shape, np.nan)
        self.bs = bs


def paged_forward(cfg, W, kv, input_ids, positions, slot_mapping, tok_seq, block_tables, last_idx, routing=None, route_log=None):
    """One iteration over T tokens of several sequences.

    input_ids, positions, slot_mapping, tok_seq: length T (tok_seq = index of the token's
    sequence within this iteration). block_tables[s]: block ids of sequence s. last_idx[s]:
    index in 0..T of the last token of sequence s. Token t at position p writes its K/V to
    slot_mapping[t] and attends to the cached positions 0..p of its sequence.
    routing (mixture-of-experts models): optional [layer][T][n_active] expert ids to use; route_log: optional list
    that receives one record per layer with the oracle's own selection and its margins.
    Returns logits [n_seq][V] of the last token of every sequence.
    """
    input_ids = np.asarray(input_ids)
    T = input_ids.size
    bs = kv.bs
    x = W["embed"][input_ids]
    for l in range(cfg["n_layers"]):
        q, k, v = _qkv(cfg, W, l, x, np.asarray(positions))
        kv.K[l][slot_mapping] = k
        kv.V[l][slot_mapping] = v
        attn = np.empty_like(q)
        for t in range(T):
            bt = np.asarray(block_tables[tok_seq[t]])
            p = np.arange(positions[t] + 1)
            slots = bt[p // bs] * bs + p % bs
            attn[t] = _attend(cfg, q[t], kv.K[l][slots], kv.V[l][slots])
        x = _post_attention(cfg, W, l, x, attn, routing, route_log)
    return _head(cfg, W, x[np.asarray(last_idx, dtype=np.int64)])


def generate_bruteforce(cfg, W, prompt, n_new, pick):
    """Autoregressive generation by the definition: recompute the whole sequence for every token.
    pick(logits, token_index) -> token id."""
    seq = list(np.asarray(prompt))
    out = []
    for i in range(n_new):
        tok = pick(forward_dense(cfg, W, seq, all_positions=False), i)
        out.append(tok)
        seq.append(tok)
    return out
