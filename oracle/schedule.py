"""Noise schedule of the chain ASD samples from (oracle side, fp64).

Test infrastructure; never imported by the product path.

The paper works with Euler chains  y_{i+1} = y_i + eta_i g(t_i, y_i) +
sigma_{i+1} xi_{i+1}  (Eq. euler-sde) and notes (Remark after Alg. 3) that a
DDPM step can be written  y_{i+1} = alpha_i y_i + beta_i E[x_0 | y_i] + noise,
with the model predicting E[x_0 | y_i].  It never prints alpha_i, beta_i.  The
reading taken here: translate the DDPM iterate to Stochastic Localization
(SL), take one SL Euler step, translate back (Sec. 3, paragraph after
Eq. euler-sde).  For the variance-preserving chain with linear beta this gives
ancestral DDPM sampling with the posterior variance, written out below; the
SL route itself is `sl_tables`, and a test checks that the two agree.

Indexing: paper step i in [0, K) moves timestep tau_i = K - i to tau_i - 1,
y_i = x_{tau_i}, y_0 ~ N(0, I).
"""
import numpy as np


def linear_beta_abar(K, beta_min=1e-4, beta_max=0.02):
    """beta[tau], abar[tau] for tau = 0..K (index 0: beta unused, abar = 1)."""
    tau = np.arange(1, K + 1, dtype=np.float64)
    if K > 1:
        beta = beta_min + (tau - 1.0) * (beta_max - beta_min) / (K - 1.0)
    else:
        beta = np.array([beta_min], dtype=np.float64)
    abar = np.concatenate([[1.0], np.cumprod(1.0 - beta)])
    return np.concatenate([[0.0], beta]), abar


def cosine_abar(K, s=0.008, beta_clip=0.999):
    """abar[tau], tau = 0..K, of the cosine noise schedule (Nichol & Dhariwal 2021): abar proportional to
    cos^2(((tau/K + s) / (1 + s)) pi / 2), each beta = 1 - abar[tau]/abar[tau-1] clipped at beta_clip (the
    unclipped last beta is 1: abar[K] = 0 would make the first model call meaningless)."""
    f = np.cos((np.arange(K + 1, dtype=np.float64) / K + s) / (1.0 + s) * np.pi / 2.0) ** 2
    beta = np.minimum(1.0 - f[1:] / f[:-1], beta_clip)
    return np.concatenate([[1.0], np.cumprod(1.0 - beta)])


def tables_from_abar(abar):
    """The same translate-to-SL / Euler step / map-back coefficients for any decreasing abar[0..K] with
    abar[0] = 1 (beta[tau] = 1 - abar[tau]/abar[tau-1]).  Returns dict(c_x, c_0, sigma, tau [K]; abar)."""
    abar = np.asarray(abar, dtype=np.float64)
    K = len(abar) - 1
    c_x, c_0, sigma = np.empty(K), np.empty(K), np.empty(K)
    tau = np.empty(K, dtype=np.int64)
    for i in range(K):
        t = K - i
        tau[i] = t
        alpha = abar[t] / abar[t - 1]
        shrink = (1.0 - abar[t - 1]) / (1.0 - abar[t])
        c_x[i] = np.sqrt(alpha) * shrink
        c_0[i] = np.sqrt(abar[t - 1]) * (1.0 - alpha) / (1.0 - abar[t])
        sigma[i] = np.sqrt((1.0 - alpha) * shrink)
    return dict(c_x=c_x, c_0=c_0, sigma=sigma, tau=tau, abar=abar)


def ddpm_tables(K, beta_min=1e-4, beta_max=0.02):
    """Per-step coefficients of  y_{i+1} = c_x y_i + c_0 D(y_i, tau_i) + sigma xi.

    Returns dict(c_x, c_0, sigma, tau [K]; abar [K+1]).  sigma[K-1] == 0.
    """
    beta, abar = linear_beta_abar(K, beta_min, beta_max)
    c_x = np.empty(K)
    c_0 = np.empty(K)
    sigma = np.empty(K)
    tau = np.empty(K, dtype=np.int64)
    for i in range(K):
        t = K - i
        tau[i] = t
        one_m = 1.0 - abar[t]
        one_m_prev = 1.0 - abar[t - 1]
        c_x[i] = np.sqrt(1.0 - beta[t]) * one_m_prev / one_m
        c_0[i] = np.sqrt(abar[t - 1]) * beta[t] / one_m
        sigma[i] = np.sqrt(beta[t] * one_m_prev / one_m)
    return dict(c_x=c_x, c_0=c_0, sigma=sigma, tau=tau, abar=abar)


def sl_time(abar):
    """SL time of a DDPM marginal: x_tau = sqrt(abar) x_0 + sqrt(1-abar) eps
    is, after scaling by sqrt(abar)/(1-abar), of the form t x_0 + sqrt(t) eps
    with t = abar/(1-abar)  (Thm. 1; OU case of the appendix, where
    exp(-s(t)) = sqrt(t/(1+t)) plays the role of sqrt(abar))."""
    return abar / (1.0 - abar)


def sl_scale(abar):
    """Factor gamma with  y^SL = gamma * x_tau."""
    return np.sqrt(abar) / (1.0 - abar)


def sl_tables(K, beta_min=1e-4, beta_max=0.02):
    """SL Euler chain equivalent to the first K-1 DDPM steps.

    Step i goes from SL time t_i to t_{i+1} with eta_i = t_{i+1} - t_i and
    noise std sqrt(eta_i) (Eq. sl-defn discretised as in Eq. euler-sde).  The
    last DDPM step (to abar = 1, t = infinity) has no SL counterpart.
    Returns dict(t [K], eta [K-1], gamma [K]).
    """
    _, abar = linear_beta_abar(K, beta_min, beta_max)
    ab = abar[K:0:-1]                 # abar at tau = K..1  <->  i = 0..K-1
    t = sl_time(ab)
    return dict(t=t, eta=np.diff(t), gamma=sl_scale(ab))
