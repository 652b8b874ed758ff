"""Pins for the schedule tables and the Gaussian-mixture posterior mean."""
import numpy as np
from scipy import integrate

from oracle import denoisers, schedule


def test_tables_against_ancestral_sampling_identities():
    K = 50
    T = schedule.ddpm_tables(K)
    beta, abar = schedule.linear_beta_abar(K)
    assert abar[0] == 1.0 and np.all(np.diff(abar) < 0)
    assert beta[1] == 1e-4 and abs(beta[K] - 0.02) < 1e-15
    assert T["sigma"][K - 1] == 0.0 and T["c_x"][K - 1] == 0.0 and abs(T["c_0"][K - 1] - 1.0) < 1e-12
    assert list(T["tau"]) == list(range(K, 0, -1))
    # If x_0 is a point mass at m, D == m and the chain must keep the forward
    # marginals: mean sqrt(abar) m, variance 1 - abar, at every level.
    m = 1.7
    for i in range(K):
        t = K - i
        mean_next = T["c_x"][i] * np.sqrt(abar[t]) * m + T["c_0"][i] * m
        var_next = T["c_x"][i] ** 2 * (1 - abar[t]) + T["sigma"][i] ** 2
        assert abs(mean_next - np.sqrt(abar[t - 1]) * m) < 1e-12
        assert abs(var_next - (1 - abar[t - 1])) < 1e-12


def test_tables_from_any_abar_keep_the_forward_marginals():
    """Cosine schedule and a random decreasing abar: a point mass at m must keep mean sqrt(abar) m and variance
    1 - abar at every level (what ancestral sampling with the posterior variance means), and the one-step
    coefficients must be one SL Euler step mapped back, as for the linear schedule."""
    rng = np.random.default_rng(5)
    K = 60
    ab_cos = schedule.cosine_abar(K)
    assert ab_cos[0] == 1.0 and np.all(np.diff(ab_cos) < 0) and ab_cos[K] > 0
    # the unclipped part of the schedule is the closed form
    f = lambda t: np.cos((t / K + 0.008) / 1.008 * np.pi / 2) ** 2
    np.testing.assert_allclose(ab_cos[1:K // 2], f(np.arange(1, K // 2)) / f(0), rtol=1e-12)
    assert abs((1 - ab_cos[K] / ab_cos[K - 1]) - 0.999) < 1e-12           # the last beta is the clipped one
    ab_rand = np.concatenate([[1.0], np.cumprod(1.0 - rng.uniform(1e-4, 0.3, K))])
    for abar in (ab_cos, ab_rand):
        T = schedule.tables_from_abar(abar)
        m = -0.9
        for i in range(K):
            t = K - i
            assert abs(T["c_x"][i] * np.sqrt(abar[t]) * m + T["c_0"][i] * m - np.sqrt(abar[t - 1]) * m) < 1e-12
            assert abs(T["c_x"][i] ** 2 * (1 - abar[t]) + T["sigma"][i] ** 2 - (1 - abar[t - 1])) < 1e-12
        ab = abar[K:0:-1]
        g, tt = schedule.sl_scale(ab), schedule.sl_time(ab)
        eta = np.diff(tt)
        np.testing.assert_allclose(g[:-1] / g[1:], T["c_x"][: K - 1], rtol=1e-9)
        np.testing.assert_allclose(eta / g[1:], T["c_0"][: K - 1], rtol=1e-9)
        np.testing.assert_allclose(np.sqrt(eta) / g[1:], T["sigma"][: K - 1], rtol=1e-9)
    # and the general routine reproduces the linear-beta tables
    _, ab_lin = schedule.linear_beta_abar(K)
    A, B = schedule.tables_from_abar(ab_lin), schedule.ddpm_tables(K)
    for k in ("c_x", "c_0", "sigma"):
        np.testing.assert_allclose(A[k], B[k], rtol=1e-12, atol=1e-15)


def test_tables_equal_one_sl_euler_step_mapped_back():
    """Translate to SL, step, map back (Sec. 3, after Eq. euler-sde):
    x' = (y + eta m + sqrt(eta) xi) / gamma' with y = gamma x  must have the
    DDPM coefficients c_x = gamma/gamma', c_0 = eta/gamma', sigma = sqrt(eta)/gamma'."""
    K = 200
    T = schedule.ddpm_tables(K)
    S = schedule.sl_tables(K)
    g, eta = S["gamma"], S["eta"]
    np.testing.assert_allclose(g[:-1] / g[1:], T["c_x"][: K - 1], rtol=1e-9)
    np.testing.assert_allclose(eta / g[1:], T["c_0"][: K - 1], rtol=1e-9)
    np.testing.assert_allclose(np.sqrt(eta) / g[1:], T["sigma"][: K - 1], rtol=1e-9)
    assert np.all(eta > 0)


def _quadrature_posterior_mean_1d(x, ab, mus, ws, s2):
    def prior(x0):
        return sum(w * np.exp(-0.5 * (x0 - m) ** 2 / s2) / np.sqrt(2 * np.pi * s2) for w, m in zip(ws, mus))

    def lik(x0):
        return np.exp(-0.5 * (x - np.sqrt(ab) * x0) ** 2 / (1 - ab))

    num = integrate.quad(lambda t: t * prior(t) * lik(t), -30, 30, points=list(mus), limit=400)[0]
    den = integrate.quad(lambda t: prior(t) * lik(t), -30, 30, points=list(mus), limit=400)[0]
    return num / den


def test_gmm_matches_quadrature_1d():
    mus = np.array([[-2.5], [0.3], [1.9]])
    ws = np.array([0.2, 0.5, 0.3])
    for ab in (0.05, 0.5, 0.9):
        for x in (-1.4, 0.2, 2.2):
            ref = _quadrature_posterior_mean_1d(x, ab, mus[:, 0], ws, 0.25)
            got = denoisers.gmm_posterior_mean([[x]], ab, mus, np.log(ws), 0.25)[0, 0]
            assert abs(got - ref) < 1e-7


def test_gmm_matches_grid_integration_2d():
    rng = np.random.default_rng(0)
    mus = 2.0 * rng.standard_normal((4, 2))
    ws = np.array([0.1, 0.2, 0.3, 0.4])
    s2, ab = 0.25, 0.6
    g = np.linspace(-9, 9, 1201)
    X0, X1 = np.meshgrid(g, g, indexing="ij")
    prior = sum(w * np.exp(-0.5 * ((X0 - m[0]) ** 2 + (X1 - m[1]) ** 2) / s2) for w, m in zip(ws, mus))
    for x in ([0.5, -1.0], [-2.0, 1.5]):
        lik = np.exp(-0.5 * ((x[0] - np.sqrt(ab) * X0) ** 2 + (x[1] - np.sqrt(ab) * X1) ** 2) / (1 - ab))
        wgt = prior * lik
        ref = np.array([(X0 * wgt).sum(), (X1 * wgt).sum()]) / wgt.sum()
        got = denoisers.gmm_posterior_mean([x], ab, mus, np.log(ws), s2)[0]
        np.testing.assert_allclose(got, ref, atol=1e-6)


def test_gmm_special_cases():
    rng = np.random.default_rng(1)
    mus = rng.standard_normal((5, 3)) * 2
    lw = np.log(np.array([0.1, 0.2, 0.3, 0.15, 0.25]))
    x = rng.standard_normal((4, 3))
    # one component: textbook Gaussian posterior mean
    ab, s2 = 0.37, 0.25
    V = ab * s2 + 1 - ab
    got = denoisers.gmm_posterior_mean(x, ab, mus[:1], [0.0], s2)
    np.testing.assert_allclose(got, mus[0] + np.sqrt(ab) * s2 / V * (x - np.sqrt(ab) * mus[0]), rtol=1e-12)
    # no noise: the observation is x_0 up to component ambiguity that vanishes with abar=1
    np.testing.assert_allclose(denoisers.gmm_posterior_mean(x, 1.0, mus[:1], [0.0], s2), x, rtol=1e-12)
    # all noise: the prior mean
    got = denoisers.gmm_posterior_mean(x, 1e-14, mus, lw, s2)
    np.testing.assert_allclose(got, np.broadcast_to(np.exp(lw) @ mus, got.shape), atol=1e-5)
    # invariance to an additive constant in log_w (unnormalised weights)
    a = denoisers.gmm_posterior_mean(x, 0.4, mus, lw, s2)
    b = denoisers.gmm_posterior_mean(x, 0.4, mus, lw + 3.3, s2)
    np.testing.assert_allclose(a, b, rtol=1e-12)
    # per-row abar equals row-by-row evaluation
    abv = np.array([0.1, 0.4, 0.7, 0.95])
    c = denoisers.gmm_posterior_mean(x, abv, mus, lw, s2)
    for n in range(4):
        np.testing.assert_allclose(c[n], denoisers.gmm_posterior_mean(x[n:n + 1], abv[n], mus, lw, s2)[0])


def test_sl_mean_is_ddpm_denoiser_under_the_map():
    """m(t, y^SL) == D(x, tau) with t = abar/(1-abar), y^SL = sqrt(abar) x/(1-abar)  (Thm. 1)."""
    rng = np.random.default_rng(2)
    mus = rng.standard_normal((6, 4)) * 2
    lw = np.log(np.full(6, 1 / 6))
    x = rng.standard_normal((5, 4)) * 1.5
    for ab in (0.02, 0.3, 0.8, 0.999):
        a = denoisers.gmm_posterior_mean(x, ab, mus, lw, 0.25)
        b = denoisers.gmm_sl_mean(schedule.sl_scale(ab) * x, schedule.sl_time(ab), mus, lw, 0.25)
        np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-11)
