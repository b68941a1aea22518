"""Parity (GPU): truncated importance weights and normalised ESS over packed sequences, through the C
ABI, against the CPU oracle.  The kernel computes in fp64: weights are compared after their rounding to
fp32 (rel 1e-6), sums and ESS values to rel 1e-11 (only the summation order differs)."""
import numpy as np
import pytest
import torch

import paper_2509_19128_amd as pl
from oracle import importance

pytestmark = pytest.mark.gpu


def _run(lp_pi, lp_mu, off, c, want_w=True):
    n_seq = len(off) - 1
    n = int(off[-1])
    d_pi = torch.from_numpy(np.asarray(lp_pi, np.float32)).cuda()
    d_mu = torch.from_numpy(np.asarray(lp_mu, np.float32)).cuda()
    d_off = torch.from_numpy(np.asarray(off, np.int64)).cuda()
    w = torch.full((max(n, 1),), float("nan"), device="cuda", dtype=torch.float32)
    sums = torch.full((n_seq, 2), float("nan"), device="cuda", dtype=torch.float64)
    ess = torch.full((n_seq,), -1.0, device="cuda", dtype=torch.float64)
    tot = torch.full((3,), float("nan"), device="cuda", dtype=torch.float64)
    pl.pl_is_ess(d_pi.data_ptr(), d_mu.data_ptr(), d_off.data_ptr(), n_seq, c, w.data_ptr() if want_w else 0,
                 sums.data_ptr(), ess.data_ptr(), tot.data_ptr(), 0)
    torch.cuda.synchronize()
    return w.cpu().numpy()[:n], sums.cpu().numpy(), ess.cpu().numpy(), tot.cpu().numpy()


def _case(rng, lens, spread):
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    n = int(off[-1])
    mu = (-rng.random(n) * 6).astype(np.float32)
    pi = (mu + rng.normal(0, spread, n)).astype(np.float32)
    return pi, mu, off


@pytest.mark.parametrize("lens,spread,c", [
    ([5], 0.5, 5.0), ([1, 1, 1], 1.0, 5.0), ([0, 7, 0, 300, 1025, 0], 0.8, 5.0), ([4096, 16384, 513, 2], 0.3, 5.0),
    ([255, 256, 257, 1023, 1024, 1025], 2.5, 5.0), ([100] * 1500, 0.7, 2.0), ([3000], 3.0, 1e9)])
def test_weights_and_ess_match_the_oracle(lens, spread, c):
    rng = np.random.default_rng(len(lens) * 1000 + int(spread * 10))
    pi, mu, off = _case(rng, lens, spread)
    w, sums, ess, tot = _run(pi, mu, off, c)
    w_ref, ess_ref, tot_ref = importance.packed_is_ess(pi, mu, off, c)
    assert np.allclose(w, w_ref, rtol=1e-6, atol=0)
    for s, L in enumerate(lens):
        seg = w_ref[off[s]:off[s + 1]]
        assert np.isclose(sums[s, 0], seg.sum(), rtol=1e-11) and np.isclose(sums[s, 1], (seg * seg).sum(), rtol=1e-11)
        if L:
            assert np.isclose(ess[s], ess_ref[s], rtol=1e-11), (s, ess[s], ess_ref[s])
        else:
            assert np.isnan(ess[s])
    assert np.isclose(tot[2], tot_ref, rtol=1e-11)
    assert np.isclose(tot[0], w_ref.sum(), rtol=1e-11) and np.isclose(tot[1], (w_ref * w_ref).sum(), rtol=1e-11)


def test_on_policy_batch_is_exactly_one_and_weights_are_optional():
    rng = np.random.default_rng(8)
    lp = (-rng.random(5000) * 9).astype(np.float32)
    off = np.array([0, 17, 17, 4000, 5000])
    w, sums, ess, tot = _run(lp, lp, off, 5.0)
    assert np.array_equal(w, np.ones(5000, np.float32))
    assert ess[0] == 1.0 and np.isnan(ess[1]) and ess[2] == 1.0 and ess[3] == 1.0 and tot[2] == 1.0
    assert tot[0] == 5000.0 and tot[1] == 5000.0
    _, sums2, ess2, tot2 = _run(lp, lp, off, 5.0, want_w=False)            # NULL weight output
    assert np.array_equal(sums, sums2) and np.array_equal(tot, tot2)


def test_runs_are_bit_reproducible_and_bad_arguments_are_rejected():
    rng = np.random.default_rng(9)
    pi, mu, off = _case(rng, [777, 12000, 31], 1.2)
    a, b = _run(pi, mu, off, 5.0), _run(pi, mu, off, 5.0)
    for x, y in zip(a, b):
        assert np.array_equal(x, y, equal_nan=True)
    t = torch.zeros(16, device="cuda", dtype=torch.float64)
    for n_seq, c in [(0, 5.0), (1, 0.0), (1, -1.0)]:
        with pytest.raises(pl.PlError) as ex:
            pl.pl_is_ess(t.data_ptr(), t.data_ptr(), t.data_ptr(), n_seq, c, 0, t.data_ptr(), t.data_ptr(), t.data_ptr(), 0)
        assert ex.value.code == pl.PL_E_INVAL


def test_engine_logprobs_rescored_under_the_same_weights_give_ess_one():
    """Closes the loop of Sec. 2.1 on the GPU path: the behaviour log-probs the engine records, fed
    back as both pi and mu (what an on-policy trainer would compute), give weights 1 and ESS 1."""
    import synth
    M = synth.CONFIGS["tiny"]
    eng = pl.Engine.from_model(M, max_batch=4, max_context=128, kv_pool_tokens=512, kv_page_tokens=32, seed=3, device=0)
    eng.load_weights(eng.pack_weights(synth.make_weights(M, seed=1235), synth.f32_to_bf16_bits))
    prompts = synth.random_prompts(np.random.default_rng(2), 4, 8, M.vocab)
    for i in range(4):
        eng.add_sequence(i, prompts[i], 20)
    lps = {i: [] for i in range(4)}
    for _ in range(8 + 20 - 1):
        o = eng.decode_step()
        for i in range(o["n"]):
            if o["emitted"][i]:
                lps[int(o["slot"][i])].append(float(o["logprob"][i]))
    eng.close()
    flat = np.concatenate([lps[i] for i in range(4)]).astype(np.float32)
    off = np.concatenate([[0], np.cumsum([len(lps[i]) for i in range(4)])])
    assert off[-1] == 80 and np.isfinite(flat).all() and (flat < 0).all()
    w, _, ess, tot = _run(flat, flat, off, 5.0)
    assert np.array_equal(w, np.ones(80, np.float32)) and np.all(ess == 1.0) and tot[2] == 1.0
