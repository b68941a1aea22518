"""Trainer-side use of the recorded behaviour log-probs (Sec. 2.1): truncated importance weights
and the normalised effective sample size.  Here only so tests can close the loop on what the
decode step records: re-scoring a sequence with the policy that produced each token gives
weights of exactly 1 and ESS exactly 1."""
import numpy as np


def truncated_is_weights(logp_current, logp_behaviour, c=5.0):
    """min(c, pi / mu) per token."""
    return np.minimum(c, np.exp(np.asarray(logp_current, np.float64) - np.asarray(logp_behaviour, np.float64)))


def normalised_ess(w):
    """(sum w)^2 / (N sum w^2)."""
    w = np.asarray(w, np.float64)
    return float(w.sum() ** 2 / (w.size * (w * w).sum()))


def packed_is_ess(logp_current, logp_behaviour, offsets, c=5.0):
    """The trainer-side reduction over a packed batch of sequences: tokens of sequence s are
    [offsets[s], offsets[s + 1]).  Returns (w, ess_seq, ess_total): the truncated weight of every
    token (Sec. 2.1: min(c, pi / mu), token level), the normalised ESS of each sequence over its own
    tokens (NaN for an empty sequence) and the normalised ESS over all tokens of the batch."""
    lp_c = np.asarray(logp_current, np.float64)
    lp_b = np.asarray(logp_behaviour, np.float64)
    off = np.asarray(offsets, np.int64)
    n = int(off[-1])
    w = np.empty(n, np.float64)
    for i in range(n):
        w[i] = min(c, np.exp(lp_c[i] - lp_b[i]))
    ess_seq = np.full(len(off) - 1, np.nan)
    for s in range(len(off) - 1):
        a, b = int(off[s]), int(off[s + 1])
        if b > a:
            s1 = 0.0
            s2 = 0.0
            for i in range(a, b):
                s1 += w[i]
                s2 += w[i] * w[i]
            ess_seq[s] = s1 * s1 / ((b - a) * s2)
    ess_total = float(w.sum() ** 2 / (n * (w * w).sum())) if n else float("nan")
    return w, ess_seq, ess_total
