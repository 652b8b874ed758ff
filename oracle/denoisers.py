"""Denoisers D(x, tau) = E[x_0 | x_tau = x] used by the oracle (fp64).

Test infrastructure; never imported by the product path.

The paper's "model call" g / the SL mean function m(t, y) (Eq. sl-defn) is
a trained network in its experiments.  The synthetic workloads replace it by
(1) the exact posterior mean of a Gaussian-mixture data law, and (2) a
random-weight residual MLP.  (1) is textbook Gaussian conjugacy and is pinned
by quadrature; (2) is not defined by the paper ("parity unpinned").
"""
import numpy as np


# --------------------------------------------------------------------------
# Gaussian mixture: x_0 ~ sum_k w_k N(mu_k, s2 I),  x_tau = sqrt(abar) x_0 + sqrt(1-abar) eps
# --------------------------------------------------------------------------
def gmm_posterior_mean(x, abar, means, log_w, s2):
    """E[x_0 | x_tau = x] for every row of x.

    x [n, d], abar scalar or [n]; means [C, d]; log_w [C]; s2 component variance.
    Marginal of component k at level abar: N(sqrt(abar) mu_k, V I) with
    V = abar s2 + 1 - abar.  Responsibility r_k is proportional to
    w_k N(x; sqrt(abar) mu_k, V I); inside component k the posterior mean is
    mu_k + (sqrt(abar) s2 / V)(x - sqrt(abar) mu_k).
    """
    x = np.atleast_2d(np.asarray(x, dtype=np.float64))
    means = np.asarray(means, dtype=np.float64)
    log_w = np.asarray(log_w, dtype=np.float64)
    abar = np.broadcast_to(np.asarray(abar, dtype=np.float64), (x.shape[0],))
    out = np.empty_like(x)
    for n in range(x.shape[0]):          # rows are independent; one at a time bounds memory
        ab = abar[n]
        V = ab * s2 + 1.0 - ab
        diff = x[n][None, :] - np.sqrt(ab) * means            # [C, d]
        logit = log_w - 0.5 * np.sum(diff * diff, axis=1) / V
        logit = logit - np.max(logit)
        r = np.exp(logit)
        r = r / np.sum(r)
        comp_mean = means + (np.sqrt(ab) * s2 / V) * diff     # [C, d]
        out[n] = r @ comp_mean
    return out


def gmm_sl_mean(y, t, means, log_w, s2):
    """SL mean function m(t, y) = E[x* | t x* + sqrt(t) xi = y] (Eq. sl-defn)
    for the same mixture.  Component k: y ~ N(t mu_k, (t^2 s2 + t) I) and
    E[x* | y, k] = mu_k + (s2 / (t s2 + 1)) (y - t mu_k)."""
    y = np.atleast_2d(np.asarray(y, dtype=np.float64))
    means = np.asarray(means, dtype=np.float64)
    log_w = np.asarray(log_w, dtype=np.float64)
    t = np.broadcast_to(np.asarray(t, dtype=np.float64), (y.shape[0],))
    out = np.empty_like(y)
    for n in range(y.shape[0]):
        tt = t[n]
        diff = y[n][None, :] - tt * means
        if tt == 0.0:                     # y_0 = 0 carries no information: prior weights
            logit = log_w.copy()
        else:
            logit = log_w - 0.5 * np.sum(diff * diff, axis=1) / (tt * tt * s2 + tt)
        logit = logit - np.max(logit)
        r = np.exp(logit)
        r = r / np.sum(r)
        out[n] = r @ (means + (s2 / (tt * s2 + 1.0)) * diff)
    return out


# --------------------------------------------------------------------------
# Residual MLP with bf16 GEMM inputs
# --------------------------------------------------------------------------
def round_to_bf16(a):
    """Round fp64 values to the nearest bf16 (ties to even), returned as fp64.

    The state is fp32 by the workload's definition, so the value is first
    rounded to fp32 and then to the top 16 bits of the fp32 pattern.
    """
    f = np.asarray(a, dtype=np.float64).astype(np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = (bits + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
    out = (rounded.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return out.astype(np.float64).reshape(np.shape(a))


def round_to_bf16_terms(a, terms):
    """An fp32 activation as it enters a matrix product: terms = 1: the nearest bf16; terms = 2: the sum of
    two bf16 numbers, the nearest bf16 of the value plus the nearest bf16 of what that left (the
    remainder is exact in fp32), i.e. 16 significant bits.  Returned as fp64."""
    hi = round_to_bf16(a)
    if terms == 1:
        return hi
    if terms != 2:
        raise ValueError("an activation is one bf16 number or the sum of two")
    a32 = np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)
    return hi + round_to_bf16(a32 - hi)


def bf16_bits_to_f64(bits):
    """uint16 bf16 patterns -> exact fp64 values."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def silu(z):
    with np.errstate(over="ignore"):      # exp(-z) = inf for very negative z gives -0.0, the right limit
        return z / (1.0 + np.exp(-z))


class MLPOracle:
    """x0hat = W_out h_n + b_out, h_0 = W_in [x ; temb(tau)] + b_in,
    h_{l+1} = h_l + SiLU(W_l h_l + b_l); the result is clipped to
    [-out_clip, out_clip] when out_clip > 0.

    Every matrix-product input is rounded just before the product -- to one bf16
    number, or (params["act_terms"] == 2) to the sum of two, see
    round_to_bf16_terms; weights are bf16; sums, bias, SiLU and the residual
    stream are fp64 here (fp32 on the device).  temb is a table [K+1, E] of bf16
    values, row tau.

    predict_eps: the network output is the noise estimate of
    x_tau = sqrt(abar) x_0 + sqrt(1 - abar) eps (the parametrisation of the
    paper's image models); x0hat = (x - sqrt(1 - abar[tau]) out) / sqrt(abar[tau]),
    then the clip.  abar is then a table indexed by tau.
    """

    def __init__(self, params, abar=None):
        self.w_in = bf16_bits_to_f64(params["w_in"])       # [W, d+E]
        self.w_blk = bf16_bits_to_f64(params["w_blk"])     # [n_blocks, W, W]
        self.w_out = bf16_bits_to_f64(params["w_out"])     # [d, W]
        self.b_in = np.asarray(params["b_in"], dtype=np.float64)
        self.b_blk = np.asarray(params["b_blk"], dtype=np.float64)
        self.b_out = np.asarray(params["b_out"], dtype=np.float64)
        self.temb = bf16_bits_to_f64(params["temb"])       # [K+1, E]
        self.out_clip = float(params.get("out_clip", 0.0))  # 0: no clipping
        self.predict_eps = bool(params.get("predict_eps", False))
        self.act_terms = int(params.get("act_terms", 1))
        self.abar = None if abar is None else np.asarray(abar, dtype=np.float64)
        if self.predict_eps and self.abar is None:
            raise ValueError("a noise-predicting network needs abar")

    def __call__(self, x, tau):
        x = np.atleast_2d(np.asarray(x, dtype=np.float64))
        tau = np.broadcast_to(np.asarray(tau, dtype=np.int64), (x.shape[0],))
        rnd = lambda v: round_to_bf16_terms(v, self.act_terms)      # noqa: E731
        inp = np.concatenate([rnd(x), self.temb[tau]], axis=1)
        h = inp @ self.w_in.T + self.b_in
        for l in range(self.w_blk.shape[0]):
            h = h + silu(rnd(h) @ self.w_blk[l].T + self.b_blk[l])
        out = rnd(h) @ self.w_out.T + self.b_out
        if self.predict_eps:
            ab = self.abar[tau][:, None]
            out = (x - np.sqrt(1.0 - ab) * out) / np.sqrt(ab)
        if self.out_clip > 0.0:            # predicted x_0 clipped to the data range
            out = np.clip(out, -self.out_clip, self.out_clip)
        return out
