"""Posterior scoring of the oracle (test infrastructure, fp64 NumPy).

Alg. 1, 'Obtain posteriors' and 'Score on active positions'; Sec. 2.2.
The lock test always uses the raw (temperature-1) posterior (Sec. 2.2, last
paragraph, and the appendix on sampling temperature).
"""
import numpy as np


def log_softmax(z):
    """log p = z - logsumexp(z) along the last axis."""
    z = np.asarray(z, dtype=np.float64)
    m = z.max(axis=-1, keepdims=True)
    return z - m - np.log(np.exp(z - m).sum(axis=-1, keepdims=True))


def kl_rows(lp_t, lp_prev):
    """D = KL(p_t || p_{t-1}) = sum_v p_t(v) (log p_t(v) - log p_{t-1}(v)), in
    nats, per row, from log-posteriors (so there is no 0 log 0 case: a
    probability that underflows contributes 0)."""
    lp_t = np.asarray(lp_t, dtype=np.float64)
    lp_prev = np.asarray(lp_prev, dtype=np.float64)
    return np.sum(np.exp(lp_t) * (lp_t - lp_prev), axis=-1)


def uncertainty(lp_t):
    """u = 1 - max_v p_t(v) per row."""
    return 1.0 - np.exp(np.max(lp_t, axis=-1))


def max_prob(lp_t):
    """max_v p_t(v) per row: the confidence UpdateMASK ranks by."""
    return np.exp(np.max(lp_t, axis=-1))


def argmax_lowest(z):
    """Index of the maximum per row; ties go to the lowest vocabulary id."""
    return np.argmax(np.asarray(z), axis=-1).astype(np.int64)
