"""Gaussian Rejection Sampler (Alg. 3) -- oracle side, fp64.

Test infrastructure; never imported by the product path.
"""
import numpy as np


def log_accept_ratio(xi, v, sigma):
    """log [ N(xi + v/sigma | 0, I) / N(xi | 0, I) ]  as Alg. 3 writes it:
    the difference of the two Gaussian log-densities."""
    shifted = xi + v / sigma
    return 0.5 * (np.dot(xi, xi) - np.dot(shifted, shifted))


def reflect(xi, m_hat, m, sigma):
    """Reject branch of Alg. 3: m + sigma (xi - 2 v <v,xi>/|v|^2), v = m_hat - m: the noise is mirrored
    across the hyperplane orthogonal to v and added to the target mean.  Requires v != 0."""
    v = m_hat - m
    return m + sigma * (xi - 2.0 * v * (np.dot(v, xi) / np.dot(v, v)))


def grs(u, xi, m_hat, m, sigma):
    """One call of Alg. 3.  Returns (x, accepted, log_ratio).

    accept iff u <= min(1, ratio)  <=>  log u <= min(0, log ratio);
    accepted: x = m_hat + sigma xi; rejected: x = m + sigma (xi - 2 v <v,xi>/|v|^2),
    the reflection of xi across the hyperplane orthogonal to v = m_hat - m.
    Requires sigma > 0.  v = 0 gives ratio 1, hence acceptance.
    """
    v = m_hat - m
    lr = log_accept_ratio(xi, v, sigma)
    if np.log(u) <= min(0.0, lr):
        return m_hat + sigma * xi, True, lr
    return reflect(xi, m_hat, m, sigma), False, lr
