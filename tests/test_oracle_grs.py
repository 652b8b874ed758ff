"""Pins for the Gaussian Rejection Sampler (Alg. 3; correctness theorem in the
appendix: output ~ N(m, sigma^2 I), P[reject] = TV(N(m_hat), N(m)))."""
import numpy as np
from scipy import special, stats

from oracle import grs


def test_log_ratio_expanded_form():
    rng = np.random.default_rng(0)
    for d in (1, 3, 64):
        xi, v = rng.standard_normal(d), rng.standard_normal(d) * 0.3
        s = 0.17
        lr = grs.log_accept_ratio(xi, v, s)
        assert abs(lr - (-(np.dot(v, xi) / s + np.dot(v, v) / (2 * s * s)))) < 1e-10 * (1 + abs(lr))


def test_reflection_is_isometry_and_involution():
    rng = np.random.default_rng(1)
    d = 16
    xi, v = rng.standard_normal(d), rng.standard_normal(d)
    m = rng.standard_normal(d)
    # force a rejection: u = 1 - tiny and v with <v,xi> > 0 so ratio < 1
    if np.dot(v, xi) < 0:
        v = -v
    x, acc, _ = grs.grs(1.0 - 1e-12, xi, m + v, m, 1.0)
    assert not acc
    refl = x - m
    assert abs(np.linalg.norm(refl) - np.linalg.norm(xi)) < 1e-12
    again = refl - 2 * v * np.dot(v, refl) / np.dot(v, v)
    np.testing.assert_allclose(again, xi, atol=1e-12)
    assert abs(np.dot(refl, v) + np.dot(xi, v)) < 1e-12          # component along v flips
    # same value written from the proposal sample: yhat - v (1 + 2 sigma <v,xi>/|v|^2)
    s = 0.4
    x2, acc2, _ = grs.grs(1.0 - 1e-12, xi, m + v, m, s)
    yhat = m + v + s * xi
    np.testing.assert_allclose(x2, yhat - v * (1 + 2 * s * np.dot(v, xi) / np.dot(v, v)), atol=1e-12)


def test_accept_returns_proposal_sample_and_v0_always_accepts():
    rng = np.random.default_rng(2)
    xi, m = rng.standard_normal(5), rng.standard_normal(5)
    x, acc, lr = grs.grs(0.999999, xi, m, m, 0.3)
    assert acc and lr == 0.0
    np.testing.assert_array_equal(x, m + 0.3 * xi)


def test_reject_probability_is_total_variation():
    rng = np.random.default_rng(3)
    n = 40000
    for d, dist, s in ((1, 0.5, 1.0), (4, 0.8, 0.5), (16, 0.1, 0.2)):
        v = rng.standard_normal(d)
        v *= dist / np.linalg.norm(v)
        m = np.zeros(d)
        rej = 0
        for _ in range(n):
            _, acc, _ = grs.grs(rng.uniform(), rng.standard_normal(d), m + v, m, s)
            rej += not acc
        tv = special.erf(dist / (2 * np.sqrt(2) * s))        # 2 Phi(|v|/(2 sigma)) - 1
        assert abs(rej / n - tv) < 4.5 * np.sqrt(tv * (1 - tv) / n)


def test_output_law_is_target_for_any_proposal():
    rng = np.random.default_rng(4)
    d, s, n = 3, 0.7, 30000
    m = np.array([0.3, -1.0, 2.0])
    m_hat = m + np.array([0.9, 0.2, -0.4])
    X = np.empty((n, d))
    for t in range(n):
        X[t], _, _ = grs.grs(rng.uniform(), rng.standard_normal(d), m_hat, m, s)
    Z = (X - m) / s
    for c in range(d):
        assert stats.kstest(Z[:, c], "norm").pvalue > 1e-3
    # along the shift direction too (where acceptance / reflection act)
    e = (m_hat - m) / np.linalg.norm(m_hat - m)
    assert stats.kstest(Z @ e, "norm").pvalue > 1e-3
    assert np.max(np.abs(np.cov(Z.T) - np.eye(d))) < 0.04
