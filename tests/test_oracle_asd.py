"""Pins for the oracle's ASD (Alg. 1 + Alg. 2) against what the paper fixes:
exactness in law (correctness theorem), the structure of a round (Lemma of the
correctness proof, worst-case round lemma), special cases that reduce to the
sequential chain, and the round-complexity theorem."""
import numpy as np
import pytest
from scipy import special, stats

import asd_workloads as W
from oracle import asd, denoisers, schedule
from oracle_helpers import chain_randoms, gmm_model, oracle_setup


def _run(cfg, seed, chain, L=None, T=None, model=None):
    if T is None:
        T, _, model = oracle_setup(cfg)
    xi, u = chain_randoms(seed, chain, cfg["K"], cfg["d"])
    y, R, rounds = asd.asd_sample(xi[0], L or cfg["L"], T["c_x"], T["c_0"], T["sigma"], model, xi, u)
    return y, R, rounds, xi, u


def test_L1_is_the_sequential_chain_value_for_value():
    cfg = W.CONFIGS[1]
    T, _, model = oracle_setup(cfg)
    for chain in range(3):
        y, R, rounds, xi, _ = _run(cfg, 0, chain, L=1, T=T, model=model)
        ys = asd.sequential_chain(xi[0], T["c_x"], T["c_0"], T["sigma"], model, xi)
        assert R == cfg["K"]
        np.testing.assert_array_equal(y, ys)


def test_constant_denoiser_accepts_everything():
    """Point-mass data: D is constant, proposal == target, v == 0.  Every slot
    is accepted except the sigma = 0 last step, which is resampled to its
    (identical) mean; the trajectory equals the sequential chain."""
    K, d = 37, 3
    T = schedule.ddpm_tables(K)
    p = dict(means=np.array([[0.5, -1.0, 2.0]]), log_w=np.zeros(1), var=0.0)
    model = gmm_model(T, p)
    xi, u = chain_randoms(5, 0, K, d)
    ys = asd.sequential_chain(xi[0], T["c_x"], T["c_0"], T["sigma"], model, xi)
    for L in (2, 5, 8, 37, 64):
        y, R, rounds = asd.asd_sample(xi[0], L, T["c_x"], T["c_0"], T["sigma"], model, xi, u)
        np.testing.assert_allclose(y, ys, rtol=0, atol=1e-13)
        assert R == -(-K // L)
        for r in rounds[:-1]:
            assert r["acc"].all()


def test_round_structure_invariants():
    cfg = W.CONFIGS[1]
    T, _, model = oracle_setup(cfg)
    K, L = cfg["K"], cfg["L"]
    for chain in range(12):
        y, R, rounds, xi, u = _run(cfg, 1, chain, T=T, model=model)
        assert -(-K // L) <= R <= -(-K // 2)
        a = 0
        for r in rounds:
            assert r["a"] == a and r["b"] == min(K, a + L)
            w = r["b"] - r["a"]
            assert r["acc"][0]                                   # slot a+1 never rejected
            assert abs(r["dot"][0]) == 0.0 and r["vv"][0] == 0.0
            assert min(2, w) <= r["a_next"] - a <= w
            n_acc = r["j"] - a
            assert r["acc"][:n_acc].all() and (n_acc == w or not r["acc"][n_acc])
            # accepted values are the drafted samples, bit for bit
            np.testing.assert_array_equal(y[a + 1: r["j"] + 1], r["yhat"][:n_acc])
            if r["r"] >= 0:
                assert r["a_next"] == r["j"] + 1 == r["r"]
                assert not np.array_equal(y[r["r"]], r["yhat"][n_acc])
                # the resampled value is the reject branch of that slot ...
                np.testing.assert_array_equal(y[r["r"]], r["z_rej"][n_acc])
                i = a + n_acc
                if T["sigma"][i] > 0:
                    # ... i.e. the target mean plus sigma times a vector of the same length as xi whose
                    # component along v = m_hat - m has changed sign (reflection of Alg. 3)
                    m_t = T["c_x"][i] * y[i] + T["c_0"][i] * r["g"][n_acc]
                    m_h = T["c_x"][i] * y[i] + T["c_0"][i] * r["g"][0]
                    refl = (y[r["r"]] - m_t) / T["sigma"][i]
                    assert abs(np.linalg.norm(refl) - np.linalg.norm(xi[i + 1])) < 1e-9
                    assert abs(np.dot(refl, m_h - m_t) + np.dot(xi[i + 1], m_h - m_t)) < 1e-9
            else:
                assert r["a_next"] == r["b"]
            # the other branch of every later-tested slot is on record too (slot a+1 has none)
            assert np.isnan(r["z_rej"][0]).all() and np.isfinite(r["z_rej"][1:]).all()
            a = r["a_next"]
        assert a == K
        # the final sigma = 0 step equals the deterministic target mean
        g = model([K - 1], y[K - 1][None])[0]
        np.testing.assert_allclose(y[K], T["c_x"][K - 1] * y[K - 1] + T["c_0"][K - 1] * g, atol=1e-13)


def test_model_call_reuse_changes_the_call_count_and_nothing_else():
    """Carrying the model value at yhat_b into the next iteration when the whole window was accepted: the
    samples are the oracle's own, value for value (the mixture denoiser evaluates row by row, so a value does
    not depend on which call computed it); first calls are made only by iteration 0 and after rejections;
    with L = 1 every window is accepted whole, so one model call per step remains -- the sequential chain's
    count -- and the trajectory is the sequential chain's."""
    cfg = W.CONFIGS[1]
    T, _, model = oracle_setup(cfg)
    K = cfg["K"]
    calls = []

    def counting(idx, rows):
        calls.append(len(idx))
        return model(idx, rows)

    for chain in range(4):
        for L in (cfg["L"], 3, K):
            xi, u = chain_randoms(4, chain, K, cfg["d"])
            y0, R0, r0 = asd.asd_sample(xi[0], L, T["c_x"], T["c_0"], T["sigma"], model, xi, u)
            del calls[:]
            y1, R1, r1 = asd.asd_sample(xi[0], L, T["c_x"], T["c_0"], T["sigma"], counting, xi, u, reuse=True)
            np.testing.assert_array_equal(y0, y1)
            assert R0 == R1 and [r["j"] for r in r0] == [r["j"] for r in r1]
            first = [r["made_first_call"] for r in r1]
            assert first[0]
            for prev, f in zip(r1[:-1], first[1:]):
                assert f == (prev["j"] < prev["b"])            # a first call only after a rejection
            # rows evaluated: one per first call; per iteration w - 1 tested slots plus yhat_b when b < K
            want = sum(first) + sum((r["b"] - r["a"] - 1) + (r["b"] < K) for r in r1)
            assert sum(calls) == want
    xi, u = chain_randoms(4, 0, K, cfg["d"])
    del calls[:]
    y, R, _ = asd.asd_sample(xi[0], 1, T["c_x"], T["c_0"], T["sigma"], counting, xi, u, reuse=True)
    assert R == K and sum(calls) == K and len(calls) == K         # y_0's call, then yhat_b of iterations 0..K-2
    np.testing.assert_array_equal(y, asd.sequential_chain(xi[0], T["c_x"], T["c_0"], T["sigma"], model, xi))


def test_worst_case_round_lemma():
    """R <= 1 + K/theta + #(rounds that advanced by at most theta - 1 steps and
    did not end at K)  -- a weaker, checkable form of the round-complexity lemma."""
    cfg = W.CONFIGS[1]
    T, _, model = oracle_setup(cfg)
    for chain in range(6):
        _, R, rounds, _, _ = _run(cfg, 2, chain, T=T, model=model)
        bad = sum(1 for r in rounds if r["a_next"] - r["a"] < cfg["L"])
        assert R <= 1 + cfg["K"] / cfg["L"] + bad


def test_window_controller_is_bounded_and_follows_the_run_length():
    """The integer controller: window within [min(4, L), L]; a string of fully accepted windows drives
    it to L, a string of early rejections to the floor; censored observations count double."""
    for L in (1, 3, 8, 64, 200):
        st = asd.window_init(L)
        assert asd.window_of(st, L) == max(min(4, L), (3 * L) // 4)
        for _ in range(40):                                  # everything accepted
            w = asd.window_of(st, L)
            assert min(4, L) <= w <= L
            st = asd.window_next(st, w, w)
        assert asd.window_of(st, L) == L
        for _ in range(40):                                  # rejected right after the forced slot
            w = asd.window_of(st, L)
            st = asd.window_next(st, w, 1)
        assert asd.window_of(st, L) == min(4, L)
    assert asd.window_next(40, 10, 10) == 40 - 10 + 20       # censored: 2 w
    assert asd.window_next(40, 10, 7) == 40 - 10 + 7


@pytest.mark.parametrize("adaptive,reuse", [(False, False), (True, False), (False, True), (True, True)])
def test_exact_in_law_gaussian_data_closed_form(adaptive, reuse):
    """Single Gaussian data law: the chain is linear-Gaussian, so Law(y_i) is
    N(mean_i, var_i) by a scalar recursion.  ASD samples must follow it -- with fixed windows, with
    windows chosen from the chain's past by the controller, and with model values carried across iterations."""
    K, d, L, n = 24, 1, 6, 3000
    T = schedule.ddpm_tables(K)
    mu, s2 = 1.5, 0.25
    p = dict(means=np.array([[mu]]), log_w=np.zeros(1), var=s2)
    model = gmm_model(T, p)
    mean, var = np.zeros(K + 1), np.ones(K + 1)
    for i in range(K):
        ab = T["abar"][T["tau"][i]]
        k = np.sqrt(ab) * s2 / (ab * s2 + 1 - ab)          # D(x) = mu + k (x - sqrt(ab) mu)
        slope = T["c_x"][i] + T["c_0"][i] * k
        mean[i + 1] = slope * mean[i] + T["c_0"][i] * (mu - k * np.sqrt(ab) * mu)
        var[i + 1] = slope ** 2 * var[i] + T["sigma"][i] ** 2
    Y = np.empty((n, K + 1))
    rej = 0
    for c in range(n):
        xi, u = chain_randoms(9, c, K, d)
        y, R, rounds = asd.asd_sample(xi[0], L, T["c_x"], T["c_0"], T["sigma"], model, xi, u, adaptive=adaptive,
                                      reuse=reuse)
        Y[c] = y[:, 0]
        rej += sum(1 for r in rounds if r["r"] >= 0 and r["r"] < K)
    assert rej > n / 4                                      # the rejection branch is exercised
    for i in (1, 5, 11, 17, 23, 24):
        z = (Y[:, i] - mean[i]) / np.sqrt(var[i])
        assert stats.kstest(z, "norm").pvalue > 1e-3, i
    # joint law: lag-one covariance  Cov(y_i, y_{i+1}) = slope_i var_i
    i = 12
    ab = T["abar"][T["tau"][i]]
    slope = T["c_x"][i] + T["c_0"][i] * np.sqrt(ab) * s2 / (ab * s2 + 1 - ab)
    c_emp = np.cov(Y[:, i], Y[:, i + 1])[0, 1]
    assert abs(c_emp - slope * var[i]) < 5 * var[i] / np.sqrt(n)


def test_exact_in_law_mixture_vs_sequential():
    """Workload-1 shape (4-component mixture, d=2, K=100, L=8): ASD samples and
    independent sequential samples agree in moments and by two-sample KS."""
    cfg = W.CONFIGS[1]
    T, _, model = oracle_setup(cfg)
    n = 500
    A = np.empty((n, 3, 2))
    S = np.empty((n, 3, 2))
    pick = [40, 80, 100]
    for c in range(n):
        y, _, _, _, _ = _run(cfg, 21, c, T=T, model=model)
        A[c] = y[pick]
        xi, _ = chain_randoms(22, c, cfg["K"], cfg["d"])
        S[c] = asd.sequential_chain(xi[0], T["c_x"], T["c_0"], T["sigma"], model, xi)[pick]
    for t in range(3):
        for k in range(2):
            assert stats.ks_2samp(A[:, t, k], S[:, t, k]).pvalue > 1e-3
            sd = np.sqrt(A[:, t, k].var() / n + S[:, t, k].var() / n)
            assert abs(A[:, t, k].mean() - S[:, t, k].mean()) < 4.5 * sd
        ca, cs = np.cov(A[:, t].T), np.cov(S[:, t].T)
        assert np.max(np.abs(ca - cs)) < 0.25 * max(1.0, np.max(np.abs(cs)))


def test_sl_coordinates_give_the_same_run():
    """Run ASD on the SL Euler chain (Eq. sl-defn / Eq. euler-sde, A=1, Bc=eta,
    sigma=sqrt(eta), g=m(t,.)) and on the DDPM tables with the same xi, u:
    same accept bits, trajectories equal under y^SL = gamma x  (Thm. 1)."""
    K, d, L = 60, 2, 8
    p = W.gmm_params(d, 4)
    T = schedule.ddpm_tables(K)
    S = schedule.sl_tables(K)
    Km = K - 1
    model_x = gmm_model(T, p)

    def model_sl(idx, rows):
        return denoisers.gmm_sl_mean(rows, S["t"][np.asarray(idx)], p["means"], p["log_w"], p["var"])

    for chain in range(4):
        xi, u = chain_randoms(4, chain, K, d)
        yx, Rx, rx = asd.asd_sample(xi[0], L, T["c_x"][:Km], T["c_0"][:Km], T["sigma"][:Km], model_x, xi, u)
        ysl, Rs, rs = asd.asd_sample(S["gamma"][0] * xi[0], L, np.ones(Km), S["eta"], np.sqrt(S["eta"]),
                                     model_sl, xi, u)
        assert Rx == Rs
        for a_, b_ in zip(rx, rs):
            assert a_["j"] == b_["j"] and np.array_equal(a_["acc"], b_["acc"])
        np.testing.assert_allclose(ysl, S["gamma"][:, None] * yx, rtol=1e-7)


def test_rejection_rate_matches_total_variation_on_own_path():
    """Law of total expectation on tested slots: E[reject bit] =
    E[ erf(|v| / (2 sqrt2 sigma)) ] with v from the oracle's own path."""
    cfg = W.CONFIGS[1]
    T, _, model = oracle_setup(cfg)
    obs = exp = var = 0.0
    hist = np.zeros(cfg["L"] + 1)
    hists = []
    for c in range(240):
        _, _, rounds, _, _ = _run(cfg, 31, c, T=T, model=model)
        for r in rounds:
            hist[r["j"] - r["a"]] += 1
            for k in range(1, r["b"] - r["a"]):
                s = T["sigma"][r["a"] + k]
                if s == 0.0:
                    continue
                tv = special.erf(np.sqrt(r["vv"][k]) / (2 * np.sqrt(2) * s))
                obs += not r["acc"][k]
                exp += tv
                var += tv * (1 - tv)
        if c % 80 == 79:
            hists.append(hist / hist.sum())
            hist = np.zeros(cfg["L"] + 1)
    assert var > 50 and abs(obs - exp) < 4.5 * np.sqrt(var)
    # accepted-prefix histogram is stable across seed blocks
    for h in hists[1:]:
        assert np.max(np.abs(h - hists[0])) < 0.08


def test_round_complexity_scaling():
    """SL chain, fixed step eta, theta = ceil((K/(beta eta d))^(1/3)): mean rounds
    grow no faster than K^(2/3) (round-complexity theorem; an upper bound with
    an unnamed constant, so a sanity check, not an equality)."""
    d, eta, beta = 2, 0.05, 4.25
    p = W.gmm_params(d, 4)
    Ks = [125, 500, 2000, 8000]
    means = []
    for K in Ks:
        L = int(np.ceil((K / (beta * eta * d)) ** (1 / 3)))
        t = np.arange(K) * eta

        def model(idx, rows, t=t):
            return denoisers.gmm_sl_mean(rows, t[np.asarray(idx)], p["means"], p["log_w"], p["var"])

        Rs = []
        for chain in range(4):
            xi, u = chain_randoms(7, chain, K, d)
            _, R, _ = asd.asd_sample(np.zeros(d), L, np.ones(K), np.full(K, eta), np.full(K, np.sqrt(eta)),
                                     model, xi, u, keep_rounds=False)
            Rs.append(R)
        means.append(np.mean(Rs))
    slope = np.polyfit(np.log(Ks), np.log(means), 1)[0]
    assert slope < 0.72
    ratio = np.array(means) / (np.array(Ks) ** (2 / 3) * (beta * d * eta) ** (1 / 3))
    assert ratio.max() < 2.0 and ratio.max() / ratio.min() < 1.3
    assert means[-1] < Ks[-1] / 10
