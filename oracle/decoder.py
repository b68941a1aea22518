"""The decoder the policy mu is parameterised by: pre-norm RMSNorm, rotary positions,
grouped-query attention, SwiGLU feed-forward, untied LM head, no biases.

The paper delegates the network to its generation engine ("Qwen 2.5 7B", Sec. 5 setup); the
shape family is fixed by the benchmark configurations.  Two evaluation orders are given:

  * `step`            - one token at one position against a stored K/V history (what a decode
                        step of Alg. 2's "generate next tokens" does);
  * `full_sequence`   - every position of a token sequence at once with a causal mask and no
                        cache (the definition the cached form must agree with).

Weights: dict of arrays named as in synth.weight_names; W is [out, in], y = x @ W.T.
"""
import numpy as np


def rmsnorm(h, g, eps):
    """h * g / sqrt(mean(h^2) + eps) over the last axis."""
    ms = np.mean(h * h, axis=-1, keepdims=True)
    return h * g / np.sqrt(ms + eps)


def rope(x, pos, theta):
    """Rotate the pairs (x_i, x_{i+hd/2}) of every head by angle pos * theta^(-2i/hd).
    x: [..., heads, hd]; pos: integer or array broadcastable to x.shape[:-2]."""
    hd = x.shape[-1]
    half = hd // 2
    inv_freq = np.asarray(theta, dtype=np.float64) ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(pos, dtype=np.float64)[..., None, None] * inv_freq
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1).astype(x.dtype)


def silu(t):
    return t / (1.0 + np.exp(-t))


def attend_one(q, K, V):
    """Attention of one new token over a history, grouped-query.
    q: [Hq, hd]; K, V: [n, Hkv, hd] (keys already rotated).  Query head h reads kv head
    h // (Hq / Hkv).  Returns [Hq, hd]."""
    Hq, hd = q.shape
    Hkv = K.shape[1]
    grp = Hq // Hkv
    out = np.empty_like(q)
    for h in range(Hq):
        kv = h // grp
        s = K[:, kv, :] @ q[h] / np.sqrt(float(hd))
        p = np.exp(s - s.max())
        p = p / p.sum()
        out[h] = p @ V[:, kv, :]
    return out


class Cache:
    """Per-sequence K/V history: lists over layers of arrays [n, Hkv, hd].  Entries stay as they
    were written: after a weight update they are the stale x-hat of Sec. 5.1."""

    def __init__(self, cfg, dtype=np.float64):
        self.k = [np.zeros((0, cfg.n_kv_heads, cfg.head_dim), dtype) for _ in range(cfg.n_layers)]
        self.v = [np.zeros((0, cfg.n_kv_heads, cfg.head_dim), dtype) for _ in range(cfg.n_layers)]

    def __len__(self):
        return self.k[0].shape[0] if self.k else 0

    def copy(self):
        c = Cache.__new__(Cache)
        c.k = [a.copy() for a in self.k]
        c.v = [a.copy() for a in self.v]
        return c


def step(cfg, W, token, pos, cache, dtype=np.float64):
    """Logits [vocab] for input `token` at position `pos` (== len(cache)); appends this
    position's rotated key and value to `cache`."""
    assert pos == len(cache) or cfg.n_layers == 0
    w = lambda n: W[n].astype(dtype, copy=False)
    h = w("embed")[token].copy()
    for l in range(cfg.n_layers):
        a = rmsnorm(h, w(f"l{l}.g1"), cfg.rms_eps)
        q = (w(f"l{l}.wq") @ a).reshape(cfg.n_q_heads, cfg.head_dim)
        k = (w(f"l{l}.wk") @ a).reshape(cfg.n_kv_heads, cfg.head_dim)
        v = (w(f"l{l}.wv") @ a).reshape(cfg.n_kv_heads, cfg.head_dim)
        q = rope(q, pos, cfg.rope_theta)
        k = rope(k, pos, cfg.rope_theta)
        cache.k[l] = np.concatenate([cache.k[l], k[None]], axis=0)
        cache.v[l] = np.concatenate([cache.v[l], v[None]], axis=0)
        o = attend_one(q, cache.k[l], cache.v[l]).reshape(-1)
        h = h + w(f"l{l}.wo") @ o
        a = rmsnorm(h, w(f"l{l}.g2"), cfg.rms_eps)
        m = silu(w(f"l{l}.wg") @ a) * (w(f"l{l}.wu") @ a)
        h = h + w(f"l{l}.wd") @ m
    a = rmsnorm(h, w("gf"), cfg.rms_eps)
    return w("lm_head") @ a


def full_sequence(cfg, W, tokens, dtype=np.float64):
    """Logits [n, vocab] for all positions of `tokens`, recomputed from scratch with a causal
    mask.  No cache, no incremental state."""
    w = lambda n: W[n].astype(dtype, copy=False)
    tokens = np.asarray(tokens)
    n = tokens.shape[0]
    pos = np.arange(n)
    grp = cfg.n_q_heads // cfg.n_kv_heads
    h = w("embed")[tokens]
    causal = np.tril(np.ones((n, n), dtype=bool))
    for l in range(cfg.n_layers):
        a = rmsnorm(h, w(f"l{l}.g1"), cfg.rms_eps)
        q = rope((a @ w(f"l{l}.wq").T).reshape(n, cfg.n_q_heads, cfg.head_dim), pos, cfg.rope_theta)
        k = rope((a @ w(f"l{l}.wk").T).reshape(n, cfg.n_kv_heads, cfg.head_dim), pos, cfg.rope_theta)
        v = (a @ w(f"l{l}.wv").T).reshape(n, cfg.n_kv_heads, cfg.head_dim)
        o = np.empty((n, cfg.n_q_heads, cfg.head_dim), dtype)
        for hq in range(cfg.n_q_heads):
            kv = hq // grp
            s = q[:, hq, :] @ k[:, kv, :].T / np.sqrt(float(cfg.head_dim))
            s = np.where(causal, s, -np.inf)
            p = np.exp(s - s.max(axis=1, keepdims=True))
            p = p / p.sum(axis=1, keepdims=True)
            o[:, hq, :] = p @ v[:, kv, :]
        h = h + o.reshape(n, -1) @ w(f"l{l}.wo").T
        a = rmsnorm(h, w(f"l{l}.g2"), cfg.rms_eps)
        m = silu(a @ w(f"l{l}.wg").T) * (a @ w(f"l{l}.wu").T)
        h = h + m @ w(f"l{l}.wd").T
    a = rmsnorm(h, w("gf"), cfg.rms_eps)
    return a @ w("lm_head").T
