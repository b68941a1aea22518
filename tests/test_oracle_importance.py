"""Pins for the packed importance-weight / ESS reduction of the oracle (Sec. 2.1): closed forms and
invariants that a dropped term, a wrong sign, a swapped operand or a wrong normaliser would break."""
import numpy as np
import pytest

from oracle import importance


def _packed(lens):
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)


def test_on_policy_data_has_unit_weights_and_ess_exactly_one():
    rng = np.random.default_rng(0)
    lp = -rng.random(50) * 8
    w, es, et = importance.packed_is_ess(lp, lp, _packed([7, 0, 20, 23]))
    assert np.array_equal(w, np.ones(50))
    assert es[0] == 1.0 and np.isnan(es[1]) and es[2] == 1.0 and es[3] == 1.0 and et == 1.0


def test_ratio_direction_and_truncation():
    # pi twice as likely as mu -> weight 2; half as likely -> 0.5; ratio e^3 ~ 20 -> clipped to c
    lp_pi = np.log([0.4, 0.1, 0.5])
    lp_mu = np.log([0.2, 0.2, 0.5 * np.exp(-3.0)])
    w, _, _ = importance.packed_is_ess(lp_pi, lp_mu, _packed([3]), c=5.0)
    assert np.allclose(w, [2.0, 0.5, 5.0], rtol=1e-15)
    w, _, _ = importance.packed_is_ess(lp_pi, lp_mu, _packed([3]), c=1.5)
    assert np.allclose(w, [1.5, 0.5, 1.5], rtol=1e-15)


@pytest.mark.parametrize("n,k,a,b", [(10, 3, 2.0, 0.5), (64, 1, 4.0, 1.0), (5, 5, 3.0, 1.0), (1000, 500, 1.25, 0.75)])
def test_two_valued_weights_closed_form(n, k, a, b):
    # k tokens of weight a, n - k of weight b: ESS = (k a + (n-k) b)^2 / (n (k a^2 + (n-k) b^2))
    lw = np.log(np.r_[np.full(k, a), np.full(n - k, b)])
    rng = np.random.default_rng(n)
    rng.shuffle(lw)
    mu = -rng.random(n)
    _, es, et = importance.packed_is_ess(mu + lw, mu, _packed([n]), c=5.0)
    want = (k * a + (n - k) * b) ** 2 / (n * (k * a * a + (n - k) * b * b))
    assert np.isclose(es[0], want, rtol=1e-13) and np.isclose(et, want, rtol=1e-13)


def test_one_dominant_weight_gives_one_over_n():
    # one token at the truncation level, the others with vanishing weight: ESS -> 1/N
    n = 16
    lp_mu = np.zeros(n)
    lp_pi = np.full(n, -700.0)
    lp_pi[5] = 10.0
    _, es, _ = importance.packed_is_ess(lp_pi, lp_mu, _packed([n]))
    assert np.isclose(es[0], 1.0 / n, rtol=1e-12)


def test_bounds_scale_invariance_and_consistency_of_the_batch_value():
    rng = np.random.default_rng(3)
    lens = [1, 17, 256, 3, 0, 99]
    off = _packed(lens)
    n = int(off[-1])
    mu = -rng.random(n) * 5
    pi = mu + rng.normal(0, 0.7, n)
    w, es, et = importance.packed_is_ess(pi, mu, off, c=5.0)
    assert w.max() <= 5.0 and w.min() > 0
    for s, L in enumerate(lens):
        if L:
            assert 1.0 / L - 1e-12 <= es[s] <= 1.0 + 1e-12             # Cauchy-Schwarz
            seg = w[off[s]:off[s + 1]]
            assert np.isclose(es[s], importance.normalised_ess(seg), rtol=1e-13)
    assert es[0] == 1.0                                                  # a single token
    assert np.isclose(et, importance.normalised_ess(w), rtol=1e-13)
    # the batch value is built from the per-sequence sums, not an average of per-sequence values
    s1 = sum(w[off[s]:off[s + 1]].sum() for s in range(len(lens)))
    s2 = sum((w[off[s]:off[s + 1]] ** 2).sum() for s in range(len(lens)))
    assert np.isclose(et, s1 * s1 / (n * s2), rtol=1e-13)
    # shifting every log-ratio by a constant (no truncation active) scales all weights: ESS unchanged
    w2, es2, et2 = importance.packed_is_ess(pi - 3.0, mu, off, c=5.0)
    assert np.allclose(w2, w * np.exp(-3.0), rtol=1e-12) or w.max() == 5.0
    untruncated = importance.packed_is_ess(pi - 3.0, mu, off, c=1e9)[2]
    assert np.isclose(untruncated, importance.packed_is_ess(pi - 6.0, mu, off, c=1e9)[2], rtol=1e-12)
    assert np.allclose(importance.truncated_is_weights(pi, mu, 5.0), w, rtol=1e-15)
