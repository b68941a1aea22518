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
