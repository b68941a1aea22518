"""Engine-level parity (GPU): the decode step with in-flight weight updates, through the C ABI, against
the CPU oracle, teacher-forced: the oracle samples, the engine is forced to the oracle's tokens, and the
per-step logits and recorded log-probs are compared (abs 2e-2 / rel 1e-2 for the bf16 engine).  Tokens
are compared bit-exactly given identical logits: the engine's own draw must equal the oracle's sampler
run on the engine's logits."""
import numpy as np
import pytest

import paper_2509_19128_amd as pl
import synth
from oracle import sampler
from oracle.engine import OracleEngine

from gpu_util import close

pytestmark = pytest.mark.gpu

ATOL, RTOL = 2e-2, 1e-2
M = synth.CONFIGS["tiny"]
SEED = 20250919


def _rounded(w):
    return {k: synth.bf16_round(v).astype(np.float64) for k, v in w.items()}


@pytest.fixture(scope="module")
def weights():
    master = synth.make_weights(M, seed=1235)
    return master, synth.perturb_weights(master, seed=1236, std=1e-3)


def _engine(max_batch=4, **kw):
    args = dict(max_batch=max_batch, max_context=128, kv_pool_tokens=max_batch * 128, kv_page_tokens=32, seed=SEED, device=0)
    args.update(kw)
    return pl.Engine.from_model(M, **args)


def _teacher_forced(weights, swap_steps, n_prompt=16, max_new=64, batch=4, n_weight_buffers=2, recompute=False):
    master, pert = weights
    versions = [master, pert]
    eng = _engine(batch, n_weight_buffers=n_weight_buffers)
    blobs = [eng.pack_weights(w, synth.f32_to_bf16_bits) for w in versions]
    eng.load_weights(blobs[0])
    orc = OracleEngine(M, _rounded(master), max_batch=batch, seed=SEED)
    prompts = synth.random_prompts(np.random.default_rng(77), batch, n_prompt, M.vocab)
    for i in range(batch):
        assert eng.add_sequence(1000 + i, prompts[i], max_new) == orc.add_sequence(1000 + i, prompts[i], max_new)
    worst = 0.0
    cur = 0
    for step in range(n_prompt + max_new - 1):
        if step in swap_steps:
            cur ^= 1
            orc.swap_weights(_rounded(versions[cur]), recompute_kv=recompute)
            flags = pl.PL_SWAP_WAIT | (pl.PL_SWAP_RECOMPUTE_KV if recompute else 0)
            assert eng.swap_weights(blobs[cur], flags=flags) == orc.version
        recs = orc.decode_step()
        forced = np.full(batch, -1, np.int32)
        for r in recs:
            forced[r.slot] = r.token
        out = eng.decode_step(forced)
        assert out["n"] == len(recs)
        logits = eng.debug_get_logits(out["n"])
        for i, r in enumerate(recs):
            assert (out["slot"][i], out["seq_id"][i], out["token"][i], out["position"][i]) == (r.slot, r.seq_id, r.token, r.position)
            assert (bool(out["emitted"][i]), bool(out["finished"][i]), out["weight_version"][i]) == (r.emitted, r.finished, r.weight_version)
            ok, err = close(logits[i], orc.last_logits[r.slot], ATOL, RTOL)
            worst = max(worst, err)
            assert ok, (step, r.slot, err)
            assert abs(out["logprob"][i] - r.logprob) <= ATOL + RTOL * abs(r.logprob), (step, r.slot)
    eng.close()
    return worst


def test_tiny_config_teacher_forced_with_one_swap_at_generated_token_32(weights):
    # all four sequences start together: generated token 32 is produced by engine step 15 + 32
    worst = _teacher_forced(weights, swap_steps={47})
    print("max |logit error|:", worst)


def test_tiny_config_many_swaps(weights):
    _teacher_forced(weights, swap_steps=set(range(8, 79, 8)))


def test_tiny_config_swap_cadence_of_the_off_policyness_study(weights):
    # Sec. 5.1: first update after 2L/g_max tokens, then every L/g_max; here L = 64 generated, g_max = 8
    _teacher_forced(weights, swap_steps={15 + 16 + 8 * i for i in range(6)})


def test_single_weight_buffer_swap_blocks_and_matches(weights):
    _teacher_forced(weights, swap_steps={30}, max_new=24, n_weight_buffers=1)


def _free_run(eng, steps, swap_at=None, blob=None):
    toks, lps, lgs = [], [], []
    for s in range(steps):
        if swap_at is not None and s == swap_at:
            eng.swap_weights(blob, flags=pl.PL_SWAP_WAIT)
        o = eng.decode_step()
        toks.append(o["token"].copy()); lps.append(o["logprob"].copy()); lgs.append(eng.debug_get_logits(o["n"]))
    return toks, lps, lgs


def test_engine_draws_equal_oracle_sampler_on_the_engines_logits(weights):
    master, _ = weights
    eng = _engine()
    eng.load_weights(eng.pack_weights(master, synth.f32_to_bf16_bits))
    prompts = synth.random_prompts(np.random.default_rng(5), 4, 6, M.vocab)
    temps = [1.0, 0.8, 1.0, 1.5]
    for i in range(4):
        eng.add_sequence((1 << 40) + i, prompts[i], 20, temps[i])
    for step in range(25):
        o = eng.decode_step()
        lg = eng.debug_get_logits(o["n"])
        for i in range(o["n"]):
            tok, lp = sampler.sample_row(lg[i], temps[i], SEED, int(o["seq_id"][i]), int(o["position"][i]))
            assert tok == o["token"][i], (step, i)
            assert abs(lp - o["logprob"][i]) <= 1e-4 * max(1.0, abs(lp))
    eng.close()


def test_swap_to_identical_weights_is_bit_identical_on_the_device(weights):
    master, _ = weights
    runs = []
    for swap_at in (None, 9):
        eng = _engine()
        blob = eng.pack_weights(master, synth.f32_to_bf16_bits)
        eng.load_weights(blob)
        prompts = synth.random_prompts(np.random.default_rng(6), 4, 5, M.vocab)
        for i in range(4):
            eng.add_sequence(i, prompts[i], 16)
        runs.append(_free_run(eng, 20, swap_at, blob.copy()))
        eng.close()
    for a, b in zip(runs[0], runs[1]):
        for x, y in zip(a, b):
            assert np.array_equal(x, y)


def test_sequence_is_independent_of_slot_and_neighbours(weights):
    master, _ = weights
    prompts = synth.random_prompts(np.random.default_rng(8), 4, 7, M.vocab)
    eng = _engine()
    eng.load_weights(eng.pack_weights(master, synth.f32_to_bf16_bits))
    for i in range(4):
        eng.add_sequence(50 + i, prompts[i], 12)
    full = _free_run(eng, 18)
    eng.close()
    solo = _engine(max_batch=1)
    solo.load_weights(solo.pack_weights(master, synth.f32_to_bf16_bits))
    solo.add_sequence(52, prompts[2], 12)
    forced_run = []
    for s in range(18):
        f = np.array([full[0][s][2]], np.int32)              # follow the batch run's tokens
        o = solo.decode_step(f)
        lg = solo.debug_get_logits(1)[0]
        ok, err = close(lg, full[2][s][2], 1e-3, 1e-3)
        assert ok, (s, err)
    solo.close()


def test_kv_cache_read_back_matches_oracle_and_write_round_trips(weights):
    master, _ = weights
    eng = _engine(max_batch=2, kv_page_tokens=32)
    eng.load_weights(eng.pack_weights(master, synth.f32_to_bf16_bits))
    orc = OracleEngine(M, _rounded(master), max_batch=2, seed=SEED)
    p = synth.random_prompts(np.random.default_rng(9), 2, 40, M.vocab)
    for i in range(2):
        eng.add_sequence(i, p[i], 8); orc.add_sequence(i, p[i], 8)
    for s in range(40):
        recs = orc.decode_step()
        f = np.full(2, -1, np.int32)
        for r in recs:
            f[r.slot] = r.token
        eng.decode_step(f)
    for layer in range(M.n_layers):
        k, v = eng.debug_read_kv(1, layer, 40)
        assert close(k, orc.slots[1].cache.k[layer], ATOL, RTOL)[0]
        assert close(v, orc.slots[1].cache.v[layer], ATOL, RTOL)[0]
    rng = np.random.default_rng(10)
    k2 = synth.bf16_round(rng.standard_normal((40, M.n_kv_heads, M.head_dim)).astype(np.float32))
    v2 = synth.bf16_round(rng.standard_normal((40, M.n_kv_heads, M.head_dim)).astype(np.float32))
    eng.debug_write_kv(0, 1, k2, v2)
    k3, v3 = eng.debug_read_kv(0, 1, 40)
    assert np.array_equal(k2, k3) and np.array_equal(v2, v3)
    k1, _ = eng.debug_read_kv(1, 1, 40)                     # the other slot's pages are untouched
    assert close(k1, orc.slots[1].cache.k[1], ATOL, RTOL)[0]
    eng.close()


def test_post_swap_steps_follow_new_weights_over_the_retained_cache(weights):
    """After a flip the engine must behave like the oracle built with the new weights and handed the
    engine's own (stale) cache contents: Sec. 5.1's mixed-policy semantics, checked on the device state."""
    master, pert = weights
    eng = _engine(max_batch=1)
    eng.load_weights(eng.pack_weights(master, synth.f32_to_bf16_bits))
    prompt = synth.random_prompts(np.random.default_rng(11), 1, 12, M.vocab)[0]
    eng.add_sequence(7, prompt, 20)
    toks = []
    for s in range(20):
        o = eng.decode_step()
        toks.append(int(o["token"][0]))
    inputs = list(prompt) + toks[11:19]                      # what positions 0..19 consumed
    fresh = OracleEngine(M, _rounded(pert), max_batch=1, seed=SEED)
    fresh.add_sequence(7, prompt, 20)
    fs = fresh.slots[0]
    for layer in range(M.n_layers):
        k, v = eng.debug_read_kv(0, layer, 20)
        fs.cache.k[layer], fs.cache.v[layer] = k.astype(np.float64), v.astype(np.float64)
    fs.inputs, fs.last_token, fs.n_emitted = inputs, toks[19], 9
    eng.swap_weights(eng.pack_weights(pert, synth.f32_to_bf16_bits), flags=pl.PL_SWAP_WAIT)
    for s in range(5):
        recs = fresh.decode_step()
        o = eng.decode_step(np.array([recs[0].token], np.int32))
        assert o["weight_version"][0] == 1
        ok, err = close(eng.debug_get_logits(1)[0], fresh.last_logits[0], ATOL, RTOL)
        assert ok, (s, err)
    eng.close()


def _forced_run(eng, orc, forced_stream, batch, steps, check_version=None):
    """Engine first, then the oracle under the weight version the engine's step reported: both consume
    the same pre-drawn forced tokens, so the order of the two calls does not matter."""
    for _ in range(steps):
        f = next(forced_stream)
        out = eng.decode_step(f)
        ver = int(out["weight_version"][0])
        assert (out["weight_version"] == ver).all()
        if check_version is not None:
            assert ver == check_version
        yield ver, out, f


def test_in_flight_update_staged_in_the_background_flips_between_two_steps(weights):
    """PL_SWAP_ASYNC, the mode the benchmark runs: the blob is copied on the side stream while steps go
    on; every step must compute wholly under the version it reports (old before the flip, new from the
    flip on, never a mixture), and once the copy is reported complete the very next step must flip.
    Alg. 2's update branch with Sec. 5.1's retained cache, checked on the device against the oracle."""
    import torch
    master, pert = weights
    batch = 4
    eng = _engine(batch)
    blobs = [eng.pack_weights(w, synth.f32_to_bf16_bits) for w in (master, pert)]
    eng.load_weights(blobs[0])
    pinned = torch.from_numpy(blobs[1].view(np.int16)).pin_memory()
    orc = OracleEngine(M, _rounded(master), max_batch=batch, seed=SEED)
    rng = np.random.default_rng(99)
    prompts = synth.random_prompts(rng, batch, 6, M.vocab)
    for i in range(batch):
        eng.add_sequence(50 + i, prompts[i], 60); orc.add_sequence(50 + i, prompts[i], 60)

    def stream():
        while True:
            yield rng.integers(0, M.vocab, batch).astype(np.int32)

    def compare(out, f):
        recs = orc.decode_step(f)
        lg = eng.debug_get_logits(out["n"])
        for i, r in enumerate(recs):
            assert out["weight_version"][i] == r.weight_version
            assert out["token"][i] == r.token
            ok, err = close(lg[i], orc.last_logits[r.slot], ATOL, RTOL)
            assert ok, (r.position, err)
            assert abs(out["logprob"][i] - r.logprob) <= ATOL + RTOL * abs(r.logprob)

    fs = stream()
    for ver, out, f in _forced_run(eng, orc, fs, batch, 8, check_version=0):
        compare(out, f)
    assert eng.swap_weights(pinned.data_ptr(), eng.weight_nbytes(), flags=pl.PL_SWAP_ASYNC) == 1
    seen = []
    for _ in range(200):                               # steps while the copy may still be in flight
        ready, active = eng.swap_poll()
        ver, out, f = next(_forced_run(eng, orc, fs, batch, 1))
        if ver == 1 and orc.version == 0:
            orc.swap_weights(_rounded(pert))           # the flip happened at this step's boundary
        compare(out, f)
        seen.append(ver)
        if ready:
            assert ver == 1, "the copy was complete before the step, so the step must have flipped"
        if ver == 1:
            break
    assert seen[-1] == 1 and seen == sorted(seen) and len(seen) < 40
    assert eng.swap_poll() == (False, 1)
    for ver, out, f in _forced_run(eng, orc, fs, batch, 6, check_version=1):
        compare(out, f)
    eng.close()


def test_buffer_that_went_inactive_can_be_poisoned_and_nothing_reads_it(weights):
    """Debugging aid: with pl_debug_set_poison the buffer that just went inactive is filled with NaN at
    the flip.  A full update cycle (two flips, so each buffer is poisoned once and reloaded once) must
    stay finite and must equal, bit for bit, the same run without the poison."""
    master, pert = weights
    runs = []
    for poison in (False, True):
        eng = _engine()
        blobs = [eng.pack_weights(w, synth.f32_to_bf16_bits) for w in (master, pert)]
        eng.load_weights(blobs[0])
        eng.debug_set_poison(poison)
        prompts = synth.random_prompts(np.random.default_rng(8), 4, 5, M.vocab)
        for i in range(4):
            eng.add_sequence(i, prompts[i], 40)
        lgs = []
        for s in range(30):
            if s in (6, 14, 22):
                eng.swap_weights(blobs[(s // 8 + 1) % 2], flags=pl.PL_SWAP_WAIT)
            o = eng.decode_step()
            lg = eng.debug_get_logits(o["n"])
            assert np.isfinite(lg).all() and np.isfinite(o["logprob"]).all(), s
            lgs.append((o["token"].copy(), o["weight_version"].copy(), lg))
        assert eng.stats()["swaps"] == 3
        runs.append(lgs)
        eng.close()
    for a, b in zip(*runs):
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])


def test_kv_pool_sized_from_free_device_memory():
    """kv_pool_tokens = 0: the pool takes what is free, capped at what the slots can ever use."""
    eng = _engine(kv_pool_tokens=0, max_context=128, kv_page_tokens=32)
    st = eng.stats()
    assert st["kv_pages_total"] == 4 * 4 and st["kv_pages_free"] == 16
    eng.close()


@pytest.mark.parametrize("name,batch,ctx", [("1p5b", 2, 48), ("7b", 2, 40), ("32b", 2, 20)])
def test_one_layer_slice_of_the_large_shapes_error_rms_below_one_percent_of_the_logit_rms(name, batch, ctx):
    """One layer + LM head at the 1.5B / 7B / 32B shapes (real head counts, widths and vocabulary), a couple
    of rows, short contexts: the oracle runs in float32 here to bound its memory."""
    m = synth.CONFIGS[name].with_layers(1)
    w = synth.make_weights(m, seed=4321)
    eng = pl.Engine.from_model(m, max_batch=batch, max_context=64, kv_pool_tokens=batch * 128, seed=SEED, device=0)
    eng.load_weights(eng.pack_weights(w, synth.f32_to_bf16_bits))
    wr = {k: synth.bf16_round(v) for k, v in w.items()}
    orc = OracleEngine(m, wr, max_batch=batch, seed=SEED, dtype=np.float32)
    prompts = synth.random_prompts(np.random.default_rng(12), batch, ctx, m.vocab)
    for i in range(batch):
        eng.add_sequence(i, prompts[i], 4); orc.add_sequence(i, prompts[i], 4)
    for s in range(ctx + 2):
        recs = orc.decode_step()
        f = np.full(batch, -1, np.int32)
        for r in recs:
            f[r.slot] = r.token
        o = eng.decode_step(f)
        if s % 8 == 0 or s >= ctx - 1:
            lg = eng.debug_get_logits(o["n"])
            for i, r in enumerate(recs):
                ref = orc.last_logits[r.slot]
                # The absolute tolerance is quoted for the tiny configuration, whose logits have rms 0.32
                # (0.02 sqrt(256)); these shapes give rms 0.78 / 1.2 / 1.4, and the bf16 rounding error of a layer
                # is proportional to the logit scale, so the absolute part is scaled by that ratio.  The
                # error rms itself must stay below 1 % of the logit rms (a wrong index or head mapping
                # gives errors of order 100 %).
                scale = max(1.0, float(ref.std()) / 0.32)
                ok, err = close(lg[i], ref, ATOL * scale, RTOL)
                assert ok, (s, i, err)
                assert float((lg[i] - ref).std()) <= 1e-2 * float(ref.std()), (s, i)
                assert abs(o["logprob"][i] - r.logprob) <= ATOL * scale + RTOL * abs(r.logprob)
    eng.close()


# ---- batched prompt reading on refill ---------------------------------------------------------------

def _kv_of(eng, slot, n_ctx):
    return [eng.debug_read_kv(slot, l, n_ctx) for l in range(M.n_layers)]


@pytest.mark.parametrize("n_prompt", [2, 5, 33, 100])
def test_batched_prefill_leaves_the_cache_of_reading_the_prompt_token_by_token(weights, n_prompt):
    """Against the oracle (which reads prompts one token per step, the definition): keys and values of
    every layer after pl_prefill, then the logits of the step that reads the last prompt token and the
    following steps.  Against the engine's own token-by-token path the cache must be bit-identical:
    the same kernels run with the same per-row operation order, only the row set differs."""
    master, _ = weights
    blob = None
    prompts = synth.random_prompts(np.random.default_rng(n_prompt), 3, n_prompt, M.vocab)
    orc = OracleEngine(M, _rounded(master), max_batch=4, seed=SEED)
    eng_b, eng_s = _engine(), _engine()
    for e in (eng_b, eng_s):
        blob = e.pack_weights(master, synth.f32_to_bf16_bits)
        e.load_weights(blob)
    for i in range(3):
        for e in (orc, eng_b, eng_s):
            assert e.add_sequence(50 + i, prompts[i], 6) == i
    for i in range(3):
        assert eng_b.prefill(i) == n_prompt - 1
    for _ in range(n_prompt - 1):
        orc.decode_step()
        eng_s.decode_step()
    for i in range(3):
        kv_b, kv_s = _kv_of(eng_b, i, n_prompt - 1), _kv_of(eng_s, i, n_prompt - 1)
        for l in range(M.n_layers):
            assert np.array_equal(kv_b[l][0], kv_s[l][0]) and np.array_equal(kv_b[l][1], kv_s[l][1]), (i, l)
            ok, err = close(kv_b[l][0], np.asarray(orc.slots[i].cache.k[l][:n_prompt - 1]), ATOL, RTOL)
            assert ok, ("K", i, l, err)
            ok, err = close(kv_b[l][1], np.asarray(orc.slots[i].cache.v[l][:n_prompt - 1]), ATOL, RTOL)
            assert ok, ("V", i, l, err)
    # the steps after it: teacher-forced against the oracle, bit-identical between the two engines
    for step in range(6):
        recs = orc.decode_step()
        forced = np.full(4, -1, np.int32)
        for r in recs:
            forced[r.slot] = r.token
        ob, os_ = eng_b.decode_step(forced), eng_s.decode_step(forced)
        lb, ls = eng_b.debug_get_logits(ob["n"]), eng_s.debug_get_logits(os_["n"])
        assert np.array_equal(lb, ls) and np.array_equal(ob["logprob"], os_["logprob"])
        for i, r in enumerate(recs):
            assert (ob["position"][i], bool(ob["emitted"][i]), bool(ob["finished"][i])) == (r.position, r.emitted, r.finished)
            ok, err = close(lb[i], orc.last_logits[r.slot], ATOL, RTOL)
            assert ok, (step, i, err)
    assert eng_b.stats()["prefill_positions"] == 3 * (n_prompt - 1)
    eng_b.close(); eng_s.close()


def test_batched_prefill_under_the_weights_active_at_admission_then_a_swap(weights):
    """A sequence admitted after an update reads its prompt under the new weights, while its
    neighbour keeps the cache computed under the old ones (Sec. 5.1)."""
    master, pert = weights
    orc = OracleEngine(M, _rounded(master), max_batch=4, seed=SEED)
    eng = _engine()
    blobs = [eng.pack_weights(w, synth.f32_to_bf16_bits) for w in (master, pert)]
    eng.load_weights(blobs[0])
    prompts = synth.random_prompts(np.random.default_rng(9), 2, 20, M.vocab)
    for e in (orc, eng):
        e.add_sequence(1, prompts[0], 30)
    eng.prefill(0)
    for _ in range(19):
        orc.decode_step()
    def both_step():
        recs = orc.decode_step()
        forced = np.full(4, -1, np.int32)
        for r in recs:
            forced[r.slot] = r.token
        out = eng.decode_step(forced)
        lg = eng.debug_get_logits(out["n"])
        for i, r in enumerate(recs):
            assert out["weight_version"][i] == r.weight_version and out["position"][i] == r.position
            ok, err = close(lg[i], orc.last_logits[r.slot], ATOL, RTOL)
            assert ok, (r.slot, r.position, err)
    for _ in range(5):
        both_step()
    orc.swap_weights(_rounded(pert))
    eng.swap_weights(blobs[1], flags=pl.PL_SWAP_WAIT)
    both_step()                                   # the flip happens at this step boundary
    for e in (orc, eng):
        e.add_sequence(2, prompts[1], 10)
    eng.prefill(1)
    for _ in range(19):                           # the oracle reads the new prompt token by token; slot 0 must wait
        seq0 = orc.slots[0]
        orc.slots[0] = None
        orc.decode_step()
        orc.slots[0] = seq0
    for _ in range(6):
        both_step()
    eng.close()


# ---- "KV cache recomputed" variant of the in-flight update (Sec. 5.1) -------------------------------

def test_swap_with_cache_recomputation_matches_the_oracle(weights):
    _teacher_forced(weights, swap_steps={20, 47}, recompute=True)
    _teacher_forced(weights, swap_steps={30}, max_new=24, n_weight_buffers=1, recompute=True)


def test_recomputed_cache_equals_the_cache_of_a_run_under_the_new_weights_from_the_start(weights):
    """What is unique: replaying the tokens under W' must leave, bit for bit, the cache an engine holds
    that read the same tokens under W' all along; with W' = W the cache must not change at all."""
    master, pert = weights
    prompts = synth.random_prompts(np.random.default_rng(21), 3, 9, M.vocab)
    eng_a, eng_b = _engine(), _engine()
    blobs = [eng_a.pack_weights(w, synth.f32_to_bf16_bits) for w in (master, pert)]
    eng_a.load_weights(blobs[0])
    eng_b.load_weights(blobs[1])
    for i in range(3):
        eng_a.add_sequence(70 + i, prompts[i], 40)
        eng_b.add_sequence(70 + i, prompts[i], 40)
    eng_a.prefill(0)                                             # one slot reads its prompt in a batched pass
    eng_b.prefill(0)
    for step in range(8):
        out = eng_a.decode_step()                                # slot 0 is already generating
        forced = np.full(4, -1, np.int32)
        forced[out["slot"]] = out["token"]
        eng_b.decode_step(forced)
    before = [_kv_of(eng_a, i, 8 if i else 16) for i in range(3)]
    eng_a.swap_weights(blobs[0], flags=pl.PL_SWAP_WAIT | pl.PL_SWAP_RECOMPUTE_KV)     # W' = W
    out = eng_a.decode_step()
    assert out["swap_stall_ms"] > 0 and eng_a.stats()["recompute_positions"] == 16 + 8 + 8
    forced = np.full(4, -1, np.int32)
    forced[out["slot"]] = out["token"]
    eng_b.decode_step(forced)
    for i in range(3):
        after = _kv_of(eng_a, i, 8 if i else 16)
        for l in range(M.n_layers):
            assert np.array_equal(before[i][l][0], after[l][0]) and np.array_equal(before[i][l][1], after[l][1])
    eng_a.swap_weights(blobs[1], flags=pl.PL_SWAP_WAIT | pl.PL_SWAP_RECOMPUTE_KV)     # now the new weights
    for step in range(4):
        out = eng_a.decode_step()
        forced = np.full(4, -1, np.int32)
        forced[out["slot"]] = out["token"]
        ob = eng_b.decode_step(forced)
        assert np.array_equal(eng_a.debug_get_logits(3), eng_b.debug_get_logits(3)), step
        assert np.array_equal(out["logprob"], ob["logprob"])
    for i in range(3):
        n = (9 if i else 17) + 4
        ka, kb = _kv_of(eng_a, i, n), _kv_of(eng_b, i, n)
        for l in range(M.n_layers):
            assert np.array_equal(ka[l][0], kb[l][0]) and np.array_equal(ka[l][1], kb[l][1]), (i, l)
    eng_a.close(); eng_b.close()


def test_prefill_of_a_partly_read_prompt_and_of_neighbours_in_other_states(weights):
    """pl_prefill picks up where token-by-token reading stopped; slots that are generating, or still
    reading their own prompt token by token, are not disturbed by another slot's passes."""
    master, _ = weights
    orc = OracleEngine(M, _rounded(master), max_batch=4, seed=SEED)
    eng = _engine()
    eng.load_weights(eng.pack_weights(master, synth.f32_to_bf16_bits))
    prompts = [synth.random_prompts(np.random.default_rng(60 + i), 1, n, M.vocab)[0] for i, n in enumerate([3, 40, 25])]
    for i in range(3):
        assert eng.add_sequence(300 + i, prompts[i], 30) == orc.add_sequence(300 + i, prompts[i], 30) == i

    def both_step():
        recs = orc.decode_step()
        forced = np.full(4, -1, np.int32)
        for r in recs:
            forced[r.slot] = r.token
        out = eng.decode_step(forced)
        lg = eng.debug_get_logits(out["n"])
        assert out["n"] == len(recs)
        for i, r in enumerate(recs):
            assert (out["slot"][i], out["position"][i], bool(out["emitted"][i])) == (r.slot, r.position, r.emitted)
            ok, err = close(lg[i], orc.last_logits[r.slot], ATOL, RTOL)
            assert ok, (r.slot, r.position, err)

    for _ in range(6):                 # slot 0 is generating by now, slots 1 and 2 are 6 tokens into their prompts
        both_step()
    assert eng.prefill(1) == 40 - 1 - 6
    s0, s2 = orc.slots[0], orc.slots[2]
    orc.slots[0] = orc.slots[2] = None # the oracle reads the rest of slot 1's prompt alone, token by token
    for _ in range(40 - 1 - 6):
        orc.decode_step()
    orc.slots[0], orc.slots[2] = s0, s2
    for _ in range(8):
        both_step()
    eng.close()


# ---- prompt reading in the background (Alg. 2 refill that does not stall the batch) ------------------

def test_background_prompt_reading_equals_the_blocking_one_and_the_oracle(weights):
    """pl_prefill_async: the refilled slot reads its prompt on a stream of its own while the other slots
    keep decoding, and joins the batch when done.  Unique: the cache it leaves is bit-identical to
    pl_prefill's, and from then on the sequence's logits are bit-identical to those of the same sequence
    in an engine that read the prompt the blocking way.  Against the oracle: per-position logits of the
    background-read sequence (a sequence's results do not depend on the step at which it joins)."""
    master, _ = weights
    n_prompt = 90
    prompts = synth.random_prompts(np.random.default_rng(31), 2, n_prompt, M.vocab)
    forced_tokens = np.random.default_rng(32).integers(0, M.vocab, 400).astype(np.int32)   # by position
    blob = None
    runs = {}
    for mode in ("blocking", "background"):
        eng = _engine(max_batch=4, max_context=256, kv_pool_tokens=4 * 256)
        blob = eng.pack_weights(master, synth.f32_to_bf16_bits)
        eng.load_weights(blob)
        eng.add_sequence(500, prompts[0][:5], 150)             # a neighbour that is decoding all along
        slot = eng.add_sequence(501, prompts[1], 40)
        if mode == "blocking":
            assert eng.prefill(slot) == n_prompt - 1
        else:
            assert eng.prefill_async(slot) == n_prompt - 1
            with pytest.raises(pl.PlError) as ex:
                eng.prefill_async(slot)
            assert ex.value.code == pl.PL_E_BUSY
        logits_by_pos, joined_at = {}, None
        for step in range(60):
            # the sequence is forced to the token drawn for the position it is about to read (ignored while
            # it is still reading its prompt), so both runs and the oracle feed it identical inputs
            forced = np.full(4, -1, np.int32)
            forced[0] = forced_tokens[step + 200]
            forced[slot] = forced_tokens[n_prompt - 1 + len(logits_by_pos)]
            out = eng.decode_step(forced)
            rows = {int(s): i for i, s in enumerate(out["slot"])}
            if slot in rows:
                if joined_at is None:
                    joined_at = step
                    kv = [eng.debug_read_kv(slot, l, n_prompt - 1) for l in range(M.n_layers)]
                i = rows[slot]
                assert out["position"][i] == n_prompt - 1 + len(logits_by_pos)
                logits_by_pos[int(out["position"][i])] = eng.debug_get_logits(out["n"])[i].copy()
            if len(logits_by_pos) >= 12:
                break
        assert joined_at is not None and len(logits_by_pos) >= 12
        assert eng.stats()["prefill_positions"] == n_prompt - 1 and eng.stats()["prefill_ms"] > 0
        runs[mode] = (kv, logits_by_pos, joined_at)
        eng.close()
    kv_a, lg_a, _ = runs["blocking"]
    kv_b, lg_b, joined = runs["background"]
    print("background reading joined the batch at step", joined)
    for l in range(M.n_layers):
        assert np.array_equal(kv_a[l][0], kv_b[l][0]) and np.array_equal(kv_a[l][1], kv_b[l][1])
    common = sorted(set(lg_a) & set(lg_b))
    assert len(common) >= 12
    for p in common:
        assert np.array_equal(lg_a[p], lg_b[p]), p
    # the oracle reads the same tokens, one per step
    orc = OracleEngine(M, _rounded(master), max_batch=1, seed=SEED)
    orc.add_sequence(501, prompts[1], 40)
    for p in range(max(common) + 1):
        f = None if p < n_prompt - 1 else np.array([forced_tokens[p]], np.int32)
        orc.decode_step(f)
        if p in lg_b:
            ok, err = close(lg_b[p], orc.last_logits[0], ATOL, RTOL)
            assert ok, (p, err)


def test_background_prompt_reading_across_an_update_and_a_retire(weights):
    """The prompt is read under the weights active when the reading was requested, even if an update
    becomes active before it ends; retiring a slot that is still reading waits for its passes.  The buffer
    that goes inactive at the flip is poisoned here: the fill must wait for the passes that still read it."""
    master, pert = weights
    prompts = synth.random_prompts(np.random.default_rng(33), 2, 70, M.vocab)
    eng = _engine(max_batch=4, max_context=256, kv_pool_tokens=4 * 256)
    blobs = [eng.pack_weights(w, synth.f32_to_bf16_bits) for w in (master, pert)]
    eng.load_weights(blobs[0])
    eng.debug_set_poison(True)
    ref = _engine(max_batch=4, max_context=256, kv_pool_tokens=4 * 256)
    ref.load_weights(blobs[0])
    for e in (eng, ref):
        e.add_sequence(1, prompts[0][:4], 100)
    a = eng.add_sequence(2, prompts[1], 20)
    eng.prefill_async(a)
    eng.swap_weights(blobs[1], flags=pl.PL_SWAP_WAIT)          # becomes active at the next step
    out = eng.decode_step()
    assert out["weight_version"][0] == 1
    for _ in range(40):
        out = eng.decode_step()
        if a in out["slot"].tolist():
            break
    assert a in out["slot"].tolist()
    b = ref.add_sequence(2, prompts[1], 20)
    ref.prefill(b)                                             # under the old weights, blocking
    for l in range(M.n_layers):
        ka, va = eng.debug_read_kv(a, l, 69)
        kb, vb = ref.debug_read_kv(b, l, 69)
        assert np.array_equal(ka, kb) and np.array_equal(va, vb)
    # a second update while a new slot is reading, then retire that slot at once
    c = eng.add_sequence(3, prompts[0], 20)
    eng.prefill_async(c)
    eng.swap_weights(blobs[0], flags=pl.PL_SWAP_ASYNC)
    eng.retire_sequence(c)
    for _ in range(5):
        out = eng.decode_step()
        assert np.isfinite(eng.debug_get_logits(out["n"])).all()
    eng.close(); ref.close()


# ---- the step replayed from a captured graph ---------------------------------------------------------

def test_steps_replayed_from_a_graph_equal_steps_launched_kernel_by_kernel(weights):
    """Every replay against the eager result, bit for bit, over a run in which the launch shape keeps
    changing (sequences finish and are refilled, so the row count varies; contexts cross the attention
    chunk; updates flip the weight buffer) and eager work of the program's own (blocking and background
    prompt reading, staging copies, synchronisations) runs between the replays."""
    master, pert = weights
    rng_p = np.random.default_rng(61)
    lens = [3, 9, 17, 30]
    prompts = [rng_p.integers(0, M.vocab, n).astype(np.int32) for n in (5, 40, 12, 70, 33, 8, 21)]
    runs = []
    for graphs in (False, True):
        eng = _engine(max_batch=4, max_context=256, kv_pool_tokens=4 * 256)
        eng.debug_set_graphs(graphs)
        blobs = [eng.pack_weights(w, synth.f32_to_bf16_bits) for w in (master, pert)]
        eng.load_weights(blobs[0])
        nxt = 0
        for i in range(4):
            eng.add_sequence(i, prompts[nxt], lens[i]); nxt += 1
        rec = []
        for step in range(70):
            if step in (11, 25, 48):
                eng.swap_weights(blobs[(step % 2)], flags=pl.PL_SWAP_WAIT)
            out = eng.decode_step()
            rec.append((out["slot"].copy(), out["token"].copy(), out["logprob"].copy(), out["weight_version"].copy(),
                        eng.debug_get_logits(out["n"])))
            for s, f in zip(out["slot"].tolist(), out["finished"].tolist()):
                if f:
                    eng.retire_sequence(s)
                    if nxt < len(prompts):
                        slot = eng.add_sequence(100 + nxt, prompts[nxt], 25)
                        if nxt % 2:
                            eng.prefill(slot)          # blocking passes between two replays
                        nxt += 1
        runs.append(rec)
        eng.close()
    assert len(runs[0]) == len(runs[1])
    shapes = set()
    for a, b in zip(*runs):
        shapes.add(len(a[0]))
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    assert len(shapes) >= 3       # the run did go through several launch shapes


def test_per_kernel_timers_count_only_the_steps_they_were_on_for(weights):
    """The benchmark switches the timers on for some steps of its window only: a step with timers launches
    its kernels one by one and counts one attention launch per layer; a replayed step records no events and
    must leave the counters alone; the tokens are the same either way."""
    master, _ = weights
    rng_p = np.random.default_rng(71)
    eng = _engine(max_batch=4)
    eng.load_weights(eng.pack_weights(master, synth.f32_to_bf16_bits))
    for i in range(4):
        eng.add_sequence(i, rng_p.integers(0, M.vocab, 6).astype(np.int32), 40)
    seen = []
    for step in range(12):
        on = step % 4 == 0
        eng.debug_set_profile(1 if on else 0)
        before = eng.stats()
        eng.decode_step()
        after = eng.stats()
        seen.append(after["attn_launches"] - before["attn_launches"])
        if on:
            assert after["attn_ms"] > before["attn_ms"] and after["attn_kv_bytes"] > before["attn_kv_bytes"]
        else:
            assert after["attn_ms"] == before["attn_ms"] and after["attn_kv_bytes"] == before["attn_kv_bytes"]
    assert seen == [M.n_layers if s % 4 == 0 else 0 for s in range(12)]
    eng.close()


def test_more_launch_shapes_than_the_graph_cache_holds(weights):
    """Row counts 1..40 in turn (more shapes than cached graphs, so the least recently used ones are dropped
    and captured again later): every step equals the eager engine's, bit for bit."""
    master, _ = weights
    runs = []
    for graphs in (False, True):
        eng = _engine(max_batch=40, max_context=64, kv_pool_tokens=40 * 64)
        eng.debug_set_graphs(graphs)
        eng.load_weights(eng.pack_weights(master, synth.f32_to_bf16_bits))
        rng = np.random.default_rng(71)
        rec = []
        for rnd in range(2):
            for k in range(40):                     # grow the batch one sequence at a time
                eng.add_sequence(1000 * rnd + k, rng.integers(0, M.vocab, 3), 60)
                o = eng.decode_step()
                rec.append((o["token"].copy(), o["logprob"].copy()))
            for s in range(40):
                eng.retire_sequence(s)
        runs.append(rec)
        eng.close()
    for a, b in zip(*runs):
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_tied_embeddings_against_the_oracle_with_an_update(weights, dtype):
    """tie_embeddings = 1: the blob carries no LM head; the engine derives it from the embedding table at
    every load and update.  Oracle: the same decoder with lm_head = embed."""
    master, pert = weights
    f32 = dtype == "f32"
    tied = [dict(w, lm_head=w["embed"]) for w in (master, pert)]
    eng = _engine(tie_embeddings=1, dtype=pl.PL_F32 if f32 else pl.PL_BF16)
    blobs = [eng.pack_weights({k: v for k, v in w.items() if k != "lm_head"}, synth.f32_to_bf16_bits) for w in tied]
    assert blobs[0].nbytes == eng.weight_nbytes()
    eng.load_weights(blobs[0])
    prep = (lambda w: {k: v.astype(np.float64) for k, v in w.items()}) if f32 else _rounded
    orc = OracleEngine(M, prep(tied[0]), max_batch=4, seed=SEED)
    prompts = synth.random_prompts(np.random.default_rng(81), 4, 6, M.vocab)
    for i in range(4):
        eng.add_sequence(i, prompts[i], 20); orc.add_sequence(i, prompts[i], 20)
    atol, rtol = (1e-4, 1e-4) if f32 else (ATOL, RTOL)
    for step in range(22):
        if step == 9:
            orc.swap_weights(prep(tied[1]))
            eng.swap_weights(blobs[1], flags=pl.PL_SWAP_WAIT)
        if step == 15:
            orc.swap_weights(prep(tied[0]))
            eng.swap_weights(blobs[0], flags=pl.PL_SWAP_ASYNC)
            while not eng.swap_poll()[0]:
                pass
        recs = orc.decode_step()
        forced = np.full(4, -1, np.int32)
        for r in recs:
            forced[r.slot] = r.token
        out = eng.decode_step(forced)
        lg = eng.debug_get_logits(out["n"])
        for i, r in enumerate(recs):
            assert out["weight_version"][i] == r.weight_version
            ok, err = close(lg[i], orc.last_logits[r.slot], atol, rtol)
            assert ok, (step, i, err)
    eng.close()
