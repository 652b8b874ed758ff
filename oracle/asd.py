"""Sequential Euler/DDPM chain and Autospeculative Decoding (oracle, fp64).

Test infrastructure; never imported by the product path.

One chain at a time, loops not vectorised, steps in the order and notation of
Alg. 1 (main loop), Alg. 2 (verifier) and Alg. 3 (GRS, in grs.py).

A chain is given by per-step tables  A[i], Bc[i], sigma[i]  and a model
g(i_list, rows):  the target transition of step i (Eq. target-dist) is
    y_{i+1} ~ N( A[i] y_i + Bc[i] g(i, y_i),  sigma[i]^2 I ).
SL / Eq. euler-sde form: A = 1, Bc = eta_i, g = m(t_i, .).
DDPM x0-prediction form (Remark after Alg. 3): A = c_x, Bc = c_0, g = E[x_0 | .].
sigma[i] is the standard deviation of the noise added by step i (it multiplies
xi_{i+1}); the paper's sigma_i / sigma_{i+1} subscripts both mean this.

Readings of the printed algorithms (each is argued in the design notes):
 * the parallel target-mean line evaluates g at the *proposal samples* yhat_i
   (the text of Sec. 3: "speculating the means ... via the proposal samples");
 * the verifier's j is the end of the all-accepted *prefix* ("advance until
   first rejection", figure caption of Sec. 3), not the largest accepted index;
 * slot a+1 has proposal mean == target mean (Lemma in the correctness
   proof), so its model value is reused, not recomputed, and it is accepted;
 * sigma[i] == 0 (last DDPM step): limit of Alg. 3 as sigma -> 0: rejected
   unless it is slot a+1, and the resampled value is the target mean.
"""
import numpy as np

from .grs import grs, reflect


def sequential_chain(y0, A, Bc, sigma, model, xi):
    """y_{i+1} = A_i y_i + Bc_i g(i, y_i) + sigma_i xi_{i+1}  (Eq. euler-sde).

    xi: array [K+1, d]; row i+1 is consumed by step i.  Returns y [K+1, d].
    """
    K = len(A)
    y = np.empty((K + 1, len(y0)))
    y[0] = y0
    for i in range(K):
        g = model([i], y[i][None, :])[0]
        y[i + 1] = A[i] * y[i] + Bc[i] * g + sigma[i] * xi[i + 1]
    return y


def near_tie(log_u, log_ratio, eps):
    """Flag for a decision too close to call across floating-point formats."""
    return abs(log_u - log_ratio) <= eps * (1.0 + abs(log_ratio) + abs(log_u))


def asd_round(y_a, a, L, A, Bc, sigma, model, xi, u, eps=1e-4, g_a=None, evaluate_end=False):
    """One iteration of the while-loop of Alg. 1 from state (a, y_a).

    Model-call reuse across iterations (the paper's accounting of "sequential network calls" implies that
    evaluations are carried over; Alg. 1 as printed makes both calls every time):
    evaluate_end: the batched call also evaluates the model at the last proposal sample yhat_b (time index
    b), returned as g_end (None when b = K: there is no step b).  If the whole window is accepted the next
    iteration starts at y_b = yhat_b, and g_end is exactly its first model call; g_a: that value, handed in
    by the caller -- the iteration then makes no model call of its own before drafting.  Nothing else
    changes: the proposal still depends on the past only, through the same function of it.

    Returns a dict with every intermediate a device implementation can be
    compared against: yhat (proposal samples for steps a+1..b), g (model
    values at slots i=a..b-1), acc (bits of slots a+1..b), log_ratio, log_u,
    dot = <v,xi>, vv = |v|^2, flagged (near-tie), j, r (index of the
    resampled step or -1), y_new (values of y_{a+1..a_next}), a_next, and
    z_rej: what every slot's step would become were the slot rejected (the
    reject branch of Alg. 3; the target mean where sigma = 0; NaN for slot a+1,
    which cannot be rejected).  A comparison that has to follow another
    implementation through a flagged near-tie decision takes the other
    branch's value from z_rej.
    """
    K = len(A)
    b = min(K, a + L)
    w = b - a
    d = len(y_a)
    # --- model call 1 (unless its value was carried over) and proposal means / samples
    carried = g_a is not None
    if not carried:
        g_a = model([a], y_a[None, :])[0]
    yhat = np.empty((w + 1, d))          # yhat[k] = \hat y_{a+k}
    m_hat = np.empty((w + 1, d))         # m_hat[k] = \hat m_{a+k}, k>=1
    yhat[0] = y_a
    for k in range(w):
        i = a + k
        m_hat[k + 1] = A[i] * yhat[k] + Bc[i] * g_a
        yhat[k + 1] = m_hat[k + 1] + sigma[i] * xi[i + 1]
    # --- model call 2: target means at the proposal samples, all slots at once
    g = np.empty((w, d))
    g[0] = g_a
    g_end = None
    if evaluate_end and b < K:
        vals = model(list(range(a + 1, b + 1)), yhat[1:w + 1])
        g[1:] = vals[:w - 1]
        g_end = vals[w - 1]
    elif w > 1:
        g[1:] = model(list(range(a + 1, b)), yhat[1:w])
    m = np.empty((w + 1, d))
    for k in range(w):
        i = a + k
        m[k + 1] = A[i] * yhat[k] + Bc[i] * g[k]
    # --- verifier: GRS on every slot
    acc = np.zeros(w, dtype=bool)
    z = np.empty((w, d))
    log_ratio = np.full(w, np.nan)
    log_u = np.full(w, np.nan)
    dot = np.zeros(w)
    vv = np.zeros(w)
    flagged = np.zeros(w, dtype=bool)
    z_rej = np.full((w, d), np.nan)
    for k in range(w):
        i = a + k
        v = m_hat[k + 1] - m[k + 1]
        dot[k] = np.dot(v, xi[i + 1])
        vv[k] = np.dot(v, v)
        if k == 0:
            acc[k] = True
            z[k] = yhat[k + 1]
        elif sigma[i] == 0.0:
            acc[k] = False
            z[k] = z_rej[k] = m[k + 1]
        else:
            z[k], acc[k], log_ratio[k] = grs(u[i + 1], xi[i + 1], m_hat[k + 1], m[k + 1], sigma[i])
            log_u[k] = np.log(u[i + 1])
            flagged[k] = near_tie(log_u[k], log_ratio[k], eps)
            z_rej[k] = reflect(xi[i + 1], m_hat[k + 1], m[k + 1], sigma[i]) if vv[k] > 0.0 else z[k]
    # --- accepted prefix
    n_acc = 0
    while n_acc < w and acc[n_acc]:
        n_acc += 1
    j = a + n_acc
    # --- advance until first rejection
    if j < b:
        y_new = z[: n_acc + 1].copy()      # y_{a+1..j+1}; the last one is the resampled value
        a_next = j + 1
        r = j + 1
    else:
        y_new = z[:n_acc].copy()
        a_next = j
        r = -1
    return dict(a=a, b=b, j=j, r=r, a_next=a_next, yhat=yhat[1:], g=g, acc=acc,
                log_ratio=log_ratio, log_u=log_u, dot=dot, vv=vv, flagged=flagged,
                y_new=y_new, z_rej=z_rej, g_end=g_end, made_first_call=not carried)


def window_init(L):
    """State of the window controller before the first round (see window_next)."""
    return 4 * L


def window_of(state, L):
    """Window length the controller asks for: three quarters of the running mean of the accepted run
    length (state / 4), within [min(4, L), L]."""
    return max(min(4, L), min(L, (3 * state) >> 4))


def window_next(state, w_used, n_acc):
    """Window controller (an extension: Alg. 1 takes the speculation length as a fixed input).

    The length of the next window may depend on the past of the chain only, which keeps every step's law
    intact (the correctness proof conditions on the past; the proposal of a round is any function of it).
    The controller tracks a running mean of the accepted run length n_acc in integers:
    state <- state - floor(state / 4) + obs,  obs = n_acc, or 2 * w_used when the whole window was
    accepted (the run was cut short by the window, so the observation is censored)."""
    obs = 2 * w_used if n_acc == w_used else n_acc
    return state - (state >> 2) + obs


def asd_sample(y0, L, A, Bc, sigma, model, xi, u, eps=1e-4, keep_rounds=True, adaptive=False, reuse=False):
    """Alg. 1.  Returns (y [K+1, d], R, rounds) with rounds the list of
    per-iteration records of `asd_round` (empty if keep_rounds is False).
    adaptive: the window of each round comes from the controller above (never longer than L).
    reuse: an iteration whose whole window is accepted hands the model value at its last sample to the next
    one (see asd_round); the samples are the same, the number of model calls is not."""
    K = len(A)
    y = np.empty((K + 1, len(y0)))
    y[0] = y0
    a = 0
    R = 0
    rounds = []
    state = window_init(L)
    g_carry = None
    while a < K:
        win = window_of(state, L) if adaptive else L
        rec = asd_round(y[a], a, win, A, Bc, sigma, model, xi, u, eps, g_a=g_carry, evaluate_end=reuse)
        g_carry = rec["g_end"] if (reuse and rec["j"] == rec["b"]) else None
        y[a + 1: rec["a_next"] + 1] = rec["y_new"]
        state = window_next(state, rec["b"] - a, rec["j"] - a)
        a = rec["a_next"]
        R += 1
        if keep_rounds:
            rounds.append(rec)
    return y, R, rounds
