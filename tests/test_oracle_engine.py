"""Pins for oracle/engine.py: the Actor-loop semantics of Alg. 2 and the stale-KV weight update of
Sec. 5.1, checked through invariants and against the cache-free recomputation."""
import numpy as np
import pytest

import synth
from oracle import decoder, importance, sampler
from oracle.engine import OracleEngine

CFG = synth.ModelCfg(n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=48, vocab=53)
SEED = 99


def _weights(seed):
    return {k: v.astype(np.float64) for k, v in synth.make_weights(CFG, seed, 0.3).items()}


W0, W1 = _weights(0), _weights(1)
PROMPTS = synth.random_prompts(np.random.default_rng(3), 4, 5, CFG.vocab)


def _run(eng, steps, swap_at=None, new_w=None, recompute=False):
    recs = []
    for s in range(steps):
        if swap_at is not None and s == swap_at:
            eng.swap_weights(new_w, recompute_kv=recompute)
        recs.append(eng.decode_step())
    return recs


def _engine(w=W0, n=3, max_new=8):
    eng = OracleEngine(CFG, w, max_batch=4, seed=SEED)
    for i in range(n):
        eng.add_sequence(100 + i, PROMPTS[i], max_new)
    return eng


def test_life_cycle_of_a_slot():
    eng = OracleEngine(CFG, W0, max_batch=2, seed=SEED)
    s = eng.add_sequence(7, PROMPTS[0], max_new=3)
    assert s == 0
    seen = []
    for step in range(5 + 3 - 1):
        (r,) = eng.decode_step()
        seen.append((r.position, r.emitted, r.finished))
    assert seen == [(0, False, False), (1, False, False), (2, False, False), (3, False, False),
                    (4, True, False), (5, True, False), (6, True, True)]
    assert len(eng.slots[0].cache) == 5 + 3 - 1
    eng.retire_sequence(0)
    assert eng.n_active() == 0 and eng.decode_step() == []
    with pytest.raises(RuntimeError):
        eng.retire_sequence(0)


def test_recorded_logprobs_rescored_without_cache_give_ess_one():
    """On-policy data has ESS exactly 1 (Sec. 2.1): re-score the emitted tokens with the cache-free
    recomputation under the same weights."""
    eng = _engine(n=1, max_new=10)
    recs = [r[0] for r in _run(eng, 5 + 10 - 1)]
    toks = list(PROMPTS[0]) + [r.token for r in recs if r.emitted]
    full = decoder.full_sequence(CFG, W0, np.array(toks[:-1]))
    lp_new = [sampler.log_softmax(full[r.position].astype(np.float32))[r.token] for r in recs if r.emitted]
    lp_old = [r.logprob for r in recs if r.emitted]
    w = importance.truncated_is_weights(lp_new, lp_old, c=5.0)
    assert np.allclose(w, 1.0, atol=1e-6)
    assert np.isclose(importance.normalised_ess(w), 1.0, atol=1e-9)
    assert np.isclose(importance.normalised_ess([1, 1, 1, 1]), 1.0)
    assert np.isclose(importance.normalised_ess([1, 0, 0, 0]), 0.25)
    assert importance.truncated_is_weights([0.0], [-10.0], c=5.0)[0] == 5.0


def test_swap_to_identical_weights_changes_nothing():
    a = _run(_engine(), 10)
    b = _run(_engine(), 10, swap_at=6, new_w={k: v.copy() for k, v in W0.items()})
    for ra, rb in zip(a, b):
        for x, y in zip(ra, rb):
            assert (x.token, x.logprob, x.position, x.emitted) == (y.token, y.logprob, y.position, y.emitted)
    assert [r[0].weight_version for r in b] == [0] * 6 + [1] * 4


def test_post_swap_steps_equal_new_weights_over_retained_cache():
    eng = _engine()
    _run(eng, 6)
    # a second engine built with the new weights and handed the old engine's state
    fresh = OracleEngine(CFG, W1, max_batch=4, seed=SEED)
    for s, seq in enumerate(eng.slots):
        if seq is not None:
            fresh.add_sequence(seq.seq_id, seq.prompt, seq.max_new)
            fs = fresh.slots[s]
            fs.cache, fs.inputs = seq.cache.copy(), list(seq.inputs)
            fs.last_token, fs.n_emitted = seq.last_token, seq.n_emitted
    eng.swap_weights(W1)
    for _ in range(4):
        for x, y in zip(eng.decode_step(), fresh.decode_step()):
            assert (x.token, x.logprob) == (y.token, y.logprob)
        for s in eng.last_logits:
            assert np.array_equal(eng.last_logits[s], fresh.last_logits[s])


def test_stale_cache_differs_from_recomputed_cache_and_both_from_no_swap():
    forced = None
    base = _engine(); stale = _engine(); recomp = _engine()
    for s in range(6):
        for e in (base, stale, recomp):
            e.decode_step()
    stale.swap_weights(W1)
    recomp.swap_weights(W1, recompute_kv=True)
    base.decode_step(); stale.decode_step(); recomp.decode_step()
    lb, ls, lr = base.last_logits[0], stale.last_logits[0], recomp.last_logits[0]
    assert not np.allclose(lb, ls) and not np.allclose(ls, lr) and not np.allclose(lb, lr)
    # the recomputed variant is the new policy run from scratch on the same tokens
    toks = np.array(recomp.slots[0].inputs)
    assert np.allclose(lr, decoder.full_sequence(CFG, W1, toks)[-1].astype(np.float32), atol=1e-5)
    # the stale variant: new weights, but keys/values of positions < 6 from the old weights
    assert np.array_equal(stale.slots[0].cache.k[0][:6], base.slots[0].cache.k[0][:6])
    assert not np.allclose(stale.slots[0].cache.k[0][6], base.slots[0].cache.k[0][6])


def test_swap_before_first_step_makes_both_variants_coincide():
    a = _engine(); b = _engine()
    a.swap_weights(W1); b.swap_weights(W1, recompute_kv=True)
    ra, rb = _run(a, 7), _run(b, 7)
    for x, y in zip(ra, rb):
        assert [(r.token, r.logprob) for r in x] == [(r.token, r.logprob) for r in y]
    c = _run(_engine(w=W1), 7)
    assert [(r.token, r.logprob) for r in ra[-1]] == [(r.token, r.logprob) for r in c[-1]]


def test_versions_constant_within_a_step_and_non_decreasing():
    eng = _engine(max_new=20)
    cadence = {4: W1, 9: W0, 13: W1}          # several updates land mid-sequence
    last = {}
    for s in range(18):
        if s in cadence:
            eng.swap_weights(cadence[s])
        recs = eng.decode_step()
        assert len({r.weight_version for r in recs}) == 1
        for r in recs:
            assert r.weight_version >= last.get(r.seq_id, 0)
            last[r.seq_id] = r.weight_version
    assert recs[0].weight_version == 3


def test_constant_batch_refill_and_independence_from_slot_and_neighbours():
    """Refill keeps the batch at H before every step; what a sequence produces depends on
    (seed, seq_id, its own tokens) only: not on its slot, its neighbours or when it was admitted."""
    rng = np.random.default_rng(5)
    H, total = 3, 7
    prompts = synth.random_prompts(rng, total, 4, CFG.vocab)
    lens = [3, 6, 2, 5, 4, 3, 2]
    eng = OracleEngine(CFG, W0, max_batch=H, seed=SEED)
    nxt, got = 0, {}
    for step in range(40):
        while eng.n_active() < H and nxt < total:
            eng.add_sequence(nxt, prompts[nxt], lens[nxt]); nxt += 1
        if eng.n_active() == 0:
            break
        if nxt < total:
            assert eng.n_active() == H
        for r in eng.decode_step():
            if r.emitted:
                got.setdefault(r.seq_id, []).append((r.token, r.logprob))
            if r.finished:
                eng.retire_sequence(r.slot)
    assert sorted(got) == list(range(total)) and [len(got[i]) for i in range(total)] == lens
    for i in (0, 4, 6):
        solo = OracleEngine(CFG, W0, max_batch=1, seed=SEED)
        solo.add_sequence(i, prompts[i], lens[i])
        alone = []
        for _ in range(4 + lens[i] - 1):
            alone += [(r.token, r.logprob) for r in solo.decode_step() if r.emitted]
        assert alone == got[i]


def test_teacher_forcing_records_forced_token_logprob_and_feeds_it_back():
    eng = _engine(n=1, max_new=4)
    forced_seq = [11, 22, 33, 44]
    out = []
    for s in range(5 + 4 - 1):
        f = np.full(4, -1)
        if s >= 4:
            f[0] = forced_seq[s - 4]
        out.append(eng.decode_step(f)[0])
    assert [r.token for r in out if r.emitted] == forced_seq
    full = decoder.full_sequence(CFG, W0, np.array(list(PROMPTS[0]) + forced_seq[:-1]))
    for r in out:
        if r.emitted:
            assert np.isclose(r.logprob, sampler.log_softmax(full[r.position].astype(np.float32))[r.token], atol=1e-6)


def test_bad_arguments():
    eng = OracleEngine(CFG, W0, max_batch=1, seed=SEED)
    with pytest.raises(ValueError):
        eng.add_sequence(1, PROMPTS[0], 4, temperature=0.0)
    eng.add_sequence(1, PROMPTS[0], 4)
    with pytest.raises(RuntimeError):
        eng.add_sequence(2, PROMPTS[1], 4)
