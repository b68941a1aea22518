"""Pins for oracle/philox.py and oracle/sampler.py (CPU only)."""
import os

import numpy as np
import pytest
import torch

from oracle import philox, sampler

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _bigint_philox(ctr, key):
    """Second implementation with Python integers, written from the round description."""
    c = list(ctr)
    k = list(key)
    for r in range(10):
        if r:
            k = [(k[0] + 0x9E3779B9) % 2**32, (k[1] + 0xBB67AE85) % 2**32]
        p0, p1 = 0xD2511F53 * c[0], 0xCD9E8D57 * c[2]
        c = [(p1 // 2**32) ^ c[1] ^ k[0], p1 % 2**32, (p0 // 2**32) ^ c[3] ^ k[1], p0 % 2**32]
    return c


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLD, "philox4x32_10_kat.txt")) if l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        got = [int(x) for x in philox.philox4x32_10(v[0:4], v[4:6])]
        assert got == v[6:10]
        assert _bigint_philox(v[0:4], v[4:6]) == v[6:10]


def test_philox_vectorised_matches_bigint():
    rng = np.random.default_rng(0)
    ctr = rng.integers(0, 2**32, size=(64, 4), dtype=np.uint64)
    key = (0x12345678, 0x9ABCDEF0)
    got = np.stack(philox.philox4x32_10([ctr[:, i] for i in range(4)], key), axis=1)
    for i in range(64):
        assert [int(x) for x in got[i]] == _bigint_philox([int(x) for x in ctr[i]], key)


def test_philox_is_injective_and_uniform():
    n = 1 << 16
    w = np.stack(philox.philox4x32_10((np.arange(n), 7, 1, 0), (5, 0)), axis=1)
    assert len({tuple(r) for r in w.tolist()}) == n           # a bijection never collides
    counts = np.bincount((w.reshape(-1) >> 24).astype(np.int64), minlength=256)
    exp = w.size / 256
    chi2 = ((counts - exp) ** 2 / exp).sum()
    assert chi2 < 255 + 5 * np.sqrt(2 * 255)


def test_sampler_bits_layout():
    b = philox.sampler_bits(seed=(3 << 32) | 9, seq_id=(1 << 40) | 77, position=123, vocab=11)
    for i in range(11):
        want = _bigint_philox([i // 4, 123, 77, 1 << 8], [9, 3])[i % 4]
        assert int(b[i]) == want


def test_uniform_is_exact_and_open_interval():
    bits = np.array([0, 1 << 9, 0xFFFFFFFF, 0x80000000], dtype=np.uint32)
    u = sampler.uniform_from_bits(bits)
    k = (bits >> 9).astype(np.int64)
    assert np.array_equal(u.astype(np.float64), (2 * k + 1) / 2.0**24)
    assert u.min() > 0 and u.max() < 1


def test_log_f32_exhaustive_over_every_uniform():
    """Every value the sampler can feed to LOG: all 2^23 uniforms, then all resulting -log u."""
    k = np.arange(1 << 23, dtype=np.int64)
    u = ((2 * k + 1).astype(np.float32)) * np.float32(2.0**-24)
    def check(x):
        got = sampler.log_f32(x)
        ref = np.log(x.astype(np.float64))
        ulp = np.spacing(np.abs(ref).astype(np.float32)).astype(np.float64)
        err = np.abs(got.astype(np.float64) - ref)
        assert np.all((err <= 1.0 * ulp) | (err <= 6e-7))      # near log(1)=0 the bound is absolute
        return got
    t = -check(u)
    assert t.min() > 0 and np.isfinite(t).all()
    g = -check(t)
    assert np.isfinite(g).all() and g.min() > -3 and g.max() < 17


def test_log_softmax_closed_forms():
    rng = np.random.default_rng(1)
    z = rng.normal(size=(5, 37)) * 3
    lp = sampler.log_softmax(z)
    assert np.allclose(np.exp(lp).sum(-1), 1.0, atol=1e-12) and (lp <= 0).all()
    assert np.allclose(sampler.log_softmax(np.zeros(4096)), -np.log(4096))
    assert np.allclose(sampler.log_softmax(z + 1234.5), lp, atol=1e-9)
    a, b = 0.3, -1.7                                           # two logits: -softplus(b - a)
    assert np.isclose(sampler.log_softmax(np.array([a, b]))[0], -np.log1p(np.exp(b - a)))
    assert np.allclose(lp, torch.log_softmax(torch.from_numpy(z), -1).numpy(), atol=1e-12)
    big = np.array([1e4, 0.0, -1e4])                           # no overflow
    assert np.isfinite(sampler.log_softmax(big)).all()


def test_gumbel_max_draws_from_softmax():
    logits = np.array([0.5, -1.0, 2.0, 0.0, 1.0, -3.0, 0.2, 1.5], dtype=np.float32)
    for temp in (1.0, 0.7):
        p = np.exp(sampler.log_softmax(logits.astype(np.float64) / np.float32(temp)))
        n = 20000
        cnt = np.zeros(8)
        for step in range(n):
            tok, lp = sampler.sample_row(logits, temp, seed=11, seq_id=5, position=step)
            cnt[tok] += 1
            if step < 50:
                assert np.isclose(lp, np.log(p[tok]), atol=1e-6)
        sig = np.sqrt(n * p * (1 - p))
        assert np.all(np.abs(cnt - n * p) < 4.5 * sig)


def test_sampler_temperature_ties_forcing_determinism():
    logits = np.array([0.0, 3.0, 1.0, 2.9], dtype=np.float32)
    toks = {sampler.sample_row(logits, 1e-3, 1, 2, s)[0] for s in range(200)}
    assert toks == {1}                                         # T -> 0 concentrates on the arg-max
    tok, lp = sampler.sample_row(logits, 1.0, 1, 2, 3, forced=2)
    assert tok == 2 and np.isclose(lp, sampler.log_softmax(logits.astype(np.float64))[2])
    a = [sampler.sample_row(logits, 1.0, 9, 4, s)[0] for s in range(64)]
    b = [sampler.sample_row(logits, 1.0, 9, 4, s)[0] for s in range(64)]
    c = [sampler.sample_row(logits, 1.0, 9, 5, s)[0] for s in range(64)]
    d = [sampler.sample_row(logits, 1.0, 10, 4, s)[0] for s in range(64)]
    assert a == b and a != c and a != d
    # exact ties go to the lowest index: identical logits and a huge gap elsewhere
    z = np.full(8, -1e30, dtype=np.float32)
    z[3] = z[6] = 0.0
    g = sampler.gumbel_from_bits(philox.sampler_bits(1, 1, 1, 8))
    want = 3 if g[3] >= g[6] else 6
    assert sampler.sample_row(z, 1.0, 1, 1, 1)[0] == want
    assert int(np.argmax(np.array([1.0, 5.0, 5.0], dtype=np.float32))) == 1
