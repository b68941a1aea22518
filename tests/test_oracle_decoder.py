"""Pins for oracle/decoder.py (CPU only): closed forms, library special cases, brute force."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth
from oracle import decoder

CFG = synth.ModelCfg(n_layers=3, d_model=48, n_q_heads=6, n_kv_heads=2, head_dim=8, d_ffn=80, vocab=61)


def _w(cfg=CFG, seed=0, std=0.2):
    w = synth.make_weights(cfg, seed, std)
    rng = np.random.default_rng(seed + 1)
    for k in w:                      # non-trivial gains so a dropped gain shows
        if w[k].ndim == 1:
            w[k] = (1 + 0.3 * rng.standard_normal(w[k].shape)).astype(np.float32)
    return {k: v.astype(np.float64) for k, v in w.items()}


def test_rmsnorm_closed_forms_and_library():
    rng = np.random.default_rng(0)
    h = rng.normal(size=(4, 32))
    g = rng.normal(size=32)
    out = decoder.rmsnorm(h, np.ones(32), 1e-6)
    ms = (h * h).mean(-1)
    assert np.allclose(np.sqrt((out * out).mean(-1)), 1 / np.sqrt(1 + 1e-6 / ms))
    assert np.allclose(decoder.rmsnorm(7.0 * h, g, 0.0), decoder.rmsnorm(h, g, 0.0))
    ref = F.rms_norm(torch.from_numpy(h), (32,), torch.from_numpy(g), 1e-6).numpy()
    assert np.allclose(decoder.rmsnorm(h, g, 1e-6), ref, atol=1e-13)


def test_rope_is_a_rotation_by_position_times_frequency():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(5, 3, 8))
    pos = np.array([0, 1, 7, 100, 16383])
    y = decoder.rope(x, pos, 1e4)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1))
    assert np.array_equal(y[0], x[0])                               # position 0: identity
    # pair (i, i + hd/2) as a complex number is multiplied by exp(1j * pos * theta^(-2i/hd))
    z = x[..., :4] + 1j * x[..., 4:]
    w = np.exp(1j * pos[:, None, None] * (1e4 ** (-np.arange(4) / 4.0)))
    assert np.allclose(y[..., :4] + 1j * y[..., 4:], z * w)
    # scores depend on the position difference only
    q, k = rng.normal(size=(1, 1, 8)), rng.normal(size=(1, 1, 8))
    s1 = (decoder.rope(q, np.array([9]), 1e4) * decoder.rope(k, np.array([4]), 1e4)).sum()
    s2 = (decoder.rope(q, np.array([109]), 1e4) * decoder.rope(k, np.array([104]), 1e4)).sum()
    assert np.isclose(s1, s2)


def test_silu():
    t = np.linspace(-20, 20, 41)
    assert decoder.silu(np.zeros(1))[0] == 0
    assert np.allclose(decoder.silu(t), F.silu(torch.from_numpy(t)).numpy(), atol=1e-14)
    assert np.isclose(decoder.silu(np.array([40.0]))[0], 40.0)


def test_attention_special_cases():
    rng = np.random.default_rng(2)
    K, V = rng.normal(size=(9, 2, 8)), rng.normal(size=(9, 2, 8))
    o = decoder.attend_one(np.zeros((6, 8)), K, V)                  # q = 0: plain mean of V
    for h in range(6):
        assert np.allclose(o[h], V[:, h // 3].mean(0))
    q = rng.normal(size=(6, 8))
    o1 = decoder.attend_one(q, K[:1], V[:1])                        # one cached token: its value
    for h in range(6):
        assert np.allclose(o1[h], V[0, h // 3])
    perm = rng.permutation(9)
    assert np.allclose(decoder.attend_one(q, K, V), decoder.attend_one(q, K[perm], V[perm]))


@pytest.mark.parametrize("hq,hkv", [(4, 4), (6, 2), (8, 1)])
def test_attention_against_library_sdpa(hq, hkv):
    rng = np.random.default_rng(3)
    n, hd = 13, 16
    q, K, V = rng.normal(size=(hq, hd)), rng.normal(size=(n, hkv, hd)), rng.normal(size=(n, hkv, hd))
    grp = hq // hkv
    tq = torch.from_numpy(q)[None, :, None, :]                              # [1, Hq, 1, hd]
    tk = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(grp, 0)[None]  # [1, Hq, n, hd]
    tv = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(grp, 0)[None]
    ref = F.scaled_dot_product_attention(tq, tk, tv)[0, :, 0, :].numpy()
    assert np.allclose(decoder.attend_one(q, K, V), ref, atol=1e-12)


def test_cached_decode_equals_recompute_from_scratch():
    W = _w()
    toks = np.random.default_rng(4).integers(0, CFG.vocab, size=12)
    full = decoder.full_sequence(CFG, W, toks)
    cache = decoder.Cache(CFG)
    for p, t in enumerate(toks):
        lg = decoder.step(CFG, W, int(t), p, cache)
        assert np.allclose(lg, full[p], rtol=1e-9, atol=1e-10)
        # brute force at every step too: the last row of a fresh recompute of the prefix
        if p in (0, 5, 11):
            assert np.allclose(lg, decoder.full_sequence(CFG, W, toks[: p + 1])[-1], rtol=1e-9, atol=1e-10)
    assert len(cache) == 12


def test_causality_and_position_dependence():
    W = _w()
    toks = np.random.default_rng(5).integers(0, CFG.vocab, size=10)
    a = decoder.full_sequence(CFG, W, toks)
    t2 = toks.copy()
    t2[7] = (t2[7] + 1) % CFG.vocab
    b = decoder.full_sequence(CFG, W, t2)
    assert np.allclose(a[:7], b[:7]) and not np.allclose(a[7:], b[7:])
    # swapping two earlier tokens changes a later position: order enters through the rotations
    t3 = toks.copy()
    t3[[1, 2]] = t3[[2, 1]]
    assert toks[1] != toks[2] and not np.allclose(a[9], decoder.full_sequence(CFG, W, t3)[9])


def test_whole_model_closed_forms():
    rng = np.random.default_rng(6)
    W0 = _w(CFG.with_layers(0))
    x = 17
    want = decoder.rmsnorm(W0["embed"][x], W0["gf"], CFG.rms_eps) @ W0["lm_head"].T
    got = decoder.step(CFG.with_layers(0), W0, x, 0, decoder.Cache(CFG.with_layers(0)))
    assert np.allclose(got, want)
    W = _w()
    for l in range(CFG.n_layers):                                   # dead residual branches
        W[f"l{l}.wo"] = np.zeros_like(W[f"l{l}.wo"])
        W[f"l{l}.wd"] = np.zeros_like(W[f"l{l}.wd"])
    want = decoder.rmsnorm(W["embed"][x], W["gf"], CFG.rms_eps) @ W["lm_head"].T
    cache = decoder.Cache(CFG)
    decoder.step(CFG, W, 5, 0, cache)
    assert np.allclose(decoder.step(CFG, W, x, 1, cache), want)


def test_one_layer_against_torch_modules():
    """A single layer assembled from torch library pieces (linear, rms_norm, sdpa, silu) in
    float64, with rotary applied through complex multiplication."""
    cfg = CFG.with_layers(1)
    W = _w(cfg, seed=9)
    toks = np.random.default_rng(7).integers(0, cfg.vocab, size=6)
    T = {k: torch.from_numpy(v) for k, v in W.items()}
    n, hd, half = len(toks), cfg.head_dim, cfg.head_dim // 2
    h = T["embed"][torch.from_numpy(toks)]
    a = F.rms_norm(h, (cfg.d_model,), T["l0.g1"], cfg.rms_eps)
    q = F.linear(a, T["l0.wq"]).view(n, cfg.n_q_heads, hd)
    k = F.linear(a, T["l0.wk"]).view(n, cfg.n_kv_heads, hd)
    v = F.linear(a, T["l0.wv"]).view(n, cfg.n_kv_heads, hd)
    ang = torch.arange(n, dtype=torch.float64)[:, None] * (cfg.rope_theta ** (-torch.arange(half, dtype=torch.float64) * 2 / hd))
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]
    def rotate(x):
        z = torch.complex(x[..., :half], x[..., half:]) * rot
        return torch.cat([z.real, z.imag], -1)
    q, k = rotate(q), rotate(k)
    grp = cfg.group
    o = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2).repeat_interleave(grp, 0)[None],
                                       v.permute(1, 0, 2).repeat_interleave(grp, 0)[None], is_causal=True)[0]
    h = h + F.linear(o.permute(1, 0, 2).reshape(n, -1), T["l0.wo"])
    a = F.rms_norm(h, (cfg.d_model,), T["l0.g2"], cfg.rms_eps)
    h = h + F.linear(F.silu(F.linear(a, T["l0.wg"])) * F.linear(a, T["l0.wu"]), T["l0.wd"])
    ref = F.linear(F.rms_norm(h, (cfg.d_model,), T["gf"], cfg.rms_eps), T["lm_head"]).numpy()
    assert np.allclose(decoder.full_sequence(cfg, W, toks), ref, rtol=1e-10, atol=1e-11)
