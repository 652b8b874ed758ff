"""Helpers of the GPU parity tests: run the library on oracle-chosen states and compare.

Decisions.  The oracle flags a tested slot whose margin |log u - rho| is within eps (1 + |rho| + |log u|)
(a "near-tie": fp32-vs-fp64 rounding of rho may put the two sides on different branches there).  On every
other slot the device must take the oracle's branch.  On a flagged slot either branch is a correct
outcome; the comparison then *follows the device*: the oracle's record holds both branches of every
slot (yhat = accepted value, z_rej = reject branch of Alg. 3), so the expected values of the branch the
device took are still the oracle's own arithmetic, and nothing is skipped.
"""
import numpy as np
import torch

import asd_workloads as W
from oracle import asd as oasd
from oracle_helpers import chain_randoms, oracle_setup
from paper_2505_03983_amd import runtime

DEV = "cuda:0"

# Tolerances (the benchmark spec): fp32 denoisers 1e-4, bf16 denoisers 2e-2, relative to the
# scale of the compared array (sup norm).
TOL = {"gmm": 1e-4, "mlp": 2e-2}
ACCEPT_CHUNK = 8      # the accept kernel examines the window eight slots at a time (see asd_accept in asd.h)


def rel_err(got, want):
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    if want.size == 0:
        return 0.0
    return float(np.max(np.abs(got - want)) / max(1.0, np.max(np.abs(want))))


def sup_rel(got, want):
    """max |got - want| / max |want|: for quantities with no natural unit scale (inner products)."""
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    if want.size == 0:
        return 0.0
    scale = float(np.max(np.abs(want)))
    return float(np.max(np.abs(got - want)) / scale) if scale > 0.0 else float(np.max(np.abs(got)))


def unclipped_scale(cfg, T, p, rec):
    """max |network output before the clip| over the rows of a round (1.0 for the exact GMM denoiser)."""
    if cfg["kind"] != "mlp" or not p.get("out_clip"):
        return 1.0
    from oracle_helpers import mlp_model
    raw = mlp_model(T, dict(p, out_clip=0.0))
    a, b = rec["a"], rec["b"]
    rows = np.concatenate([rec["yhat"][: b - a - 1]]) if b - a > 1 else rec["yhat"][:0]
    if rows.shape[0] == 0:
        return 1.0
    return float(np.abs(raw(list(range(a + 1, b)), rows)).max())


def oracle_chain(cfg, T, model, seed, chain, eps, L=None, K=None, adaptive=False):
    K = K or cfg["K"]
    xi, u = chain_randoms(seed, chain, K, cfg["d"])
    y, R, rounds = oasd.asd_sample(xi[0], L or cfg["L"], T["c_x"][:K], T["c_0"][:K], T["sigma"][:K], model, xi, u,
                                   eps=eps, adaptive=adaptive)
    return y, R, rounds, xi, u


def teacher_forced_round(ctx, cfg, states, L=None):
    """states: list over chains of (a, y_a) (a may equal K for a finished chain).
    Runs draft -> verify -> accept on the device from these states and returns
    dict(traj, a_next, accepted, x0hat, stats) as numpy."""
    B, K, d = ctx.chains, ctx.K, ctx.d
    L = L or ctx.L
    traj = torch.zeros((B, K + 1, d), dtype=torch.float32, device=DEV)
    a = torch.zeros(B, dtype=torch.int32, device=DEV)
    a_host = np.array([s[0] for s in states], dtype=np.int32)
    th = np.zeros((B, K + 1, d), dtype=np.float32)
    for c, (ac, ya) in enumerate(states):
        th[c, ac] = ya
    traj.copy_(torch.from_numpy(th))
    a.copy_(torch.from_numpy(a_host))
    x0hat = torch.zeros((B, L, d), dtype=torch.float32, device=DEV)
    accepted = torch.zeros(B, dtype=torch.int32, device=DEV)
    stats = torch.zeros((B, L, 4), dtype=torch.float32, device=DEV)
    ctx.draft(traj, a)
    ctx.verify(traj, a, x0hat)
    drafted = traj.cpu().numpy().copy()
    ctx.accept(traj, a, x0hat, accepted, stats)
    torch.cuda.synchronize()
    return dict(traj=traj.cpu().numpy(), drafted=drafted, a_next=a.cpu().numpy(), accepted=accepted.cpu().numpy(),
                x0hat=x0hat.cpu().numpy(), stats=stats.cpu().numpy())


def prefix_is_explained(rec, n_dev):
    """Does the device's accepted-prefix length n_dev differ from the oracle's only through flagged decisions?
    Every slot the device accepted must be accepted or flagged in the oracle's record, and the slot it
    rejected (if any) rejected or flagged."""
    w = rec["b"] - rec["a"]
    if not 1 <= n_dev <= w:
        return False
    acc, fl = rec["acc"], rec["flagged"]
    for k in range(n_dev):
        if not acc[k] and not fl[k]:
            return False
    return n_dev == w or (not acc[n_dev]) or bool(fl[n_dev])


def outcome(rec, n_acc):
    """(y_{a+1..a_next}, a_next) of the round when the accepted prefix has n_acc slots: advance rule of Alg. 1
    on the oracle's own values of both branches."""
    a, w = rec["a"], rec["b"] - rec["a"]
    if n_acc < w:
        return np.concatenate([rec["yhat"][:n_acc], rec["z_rej"][n_acc][None]]), a + n_acc + 1
    return rec["yhat"][:w].copy(), a + w


def compare_round(out, c, rec, tol, K, c_0=None, x0_scale=1.0, worst=None, xi=None):
    """Compare device results of chain c with the oracle's record of the same round; asserts on everything.
    c_0: the schedule's table (then the accept test's quantities in out["stats"] are compared too);
    xi [K+1, d]: the chain's normals, which give <v, xi> its scale |v| |xi| (the sum itself cancels).
    Returns True when the device took the oracle's own branch everywhere, False when it took the other
    branch of a flagged slot (the values are then compared on that branch).
    worst: optional dict collecting the largest errors seen, for the log."""
    a, b = rec["a"], rec["b"]
    w = b - a

    def note(key, e):
        if worst is not None:
            worst[key] = max(worst.get(key, 0.0), float(e))

    # proposal samples
    e = rel_err(out["drafted"][c][a + 1: b + 1], rec["yhat"])
    note("yhat", e)
    assert e <= tol, ("yhat", c, a, e)
    # model values at slots 0..w-1: the values the accept test consumes, at the plain bar
    e = rel_err(out["x0hat"][c][:w], rec["g"])
    note("x0hat", e)
    assert e <= tol, ("x0hat", c, a, e)
    # second bar for a clipped network: its rounding noise lives on the scale of the *unclipped* output
    # (x0_scale = max |unclipped oracle output| over these rows), far below the first bar when that scale is large
    if x0_scale > 1.0:
        note("x0hat/unclipped scale", e / x0_scale)
        assert e / x0_scale <= 5e-3, ("x0hat relative to the unclipped scale", c, a, e / x0_scale)
    # decisions: exact off flagged near-ties, walking the prefix as Alg. 2 does
    n_dev = int(out["accepted"][c])
    n_acc = rec["j"] - a
    assert prefix_is_explained(rec, n_dev), ("prefix", c, a, n_dev, n_acc, rec["flagged"][: max(n_dev, n_acc) + 1])
    # the accept test's own quantities on every examined slot (Alg. 3's ratio line)
    if c_0 is not None and "stats" in out and w > 1:
        hi = min(w, ACCEPT_CHUNK * (min(n_dev, w - 1) // ACCEPT_CHUNK + 1))
        st = np.asarray(out["stats"][c][:hi], dtype=np.float64)
        ks = np.arange(1, hi)
        c0 = np.asarray(c_0, dtype=np.float64)[a + ks]
        live = np.isfinite(rec["log_ratio"][ks])            # sigma = 0 slots have no ratio
        if xi is not None and live.any():
            cs = np.sqrt(rec["vv"][ks]) * np.linalg.norm(np.asarray(xi)[a + ks + 1], axis=1)     # Cauchy-Schwarz scale
            e_dot = float(np.max(np.abs(c0 * st[ks, 0] - rec["dot"][ks])[live]) / max(np.max(cs[live]), 1e-300))
        else:
            e_dot = sup_rel((c0 * st[ks, 0])[live], rec["dot"][ks][live])
        e_vv = sup_rel((c0 * c0 * st[ks, 1])[live], rec["vv"][ks][live])
        note("<v,xi>", e_dot)
        note("|v|^2", e_vv)
        assert e_dot <= tol and e_vv <= tol, ("accept sums", c, a, e_dot, e_vv)
        lu, rho = rec["log_u"][ks][live], rec["log_ratio"][ks][live]
        e_lu = np.max(np.abs(st[ks, 2][live] - lu) / (1.0 + np.abs(lu))) if live.any() else 0.0
        # the bar on rho is the premise of the near-tie flag: an error below eps (1 + |rho| + |log u|)
        e_rho = np.max(np.abs(st[ks, 3][live] - rho) / (1.0 + np.abs(rho) + np.abs(lu))) if live.any() else 0.0
        note("log u", e_lu)
        note("rho", e_rho)
        assert e_lu <= 2e-6, ("log u", c, a, e_lu)
        assert e_rho <= tol, ("rho", c, a, e_rho)
    # values written by the round, on the branch the device took
    y_new, a_next = outcome(rec, n_dev)
    assert out["a_next"][c] == a_next, ("a_next", c, a, out["a_next"][c], a_next)
    e = rel_err(out["traj"][c][a + 1: a_next + 1], y_new)
    note("y_new", e)
    assert e <= tol, ("y_new", c, a, e)
    return n_dev == n_acc


def follow_chain(cfg, T, model, seed, c, tj, tol, L=None, adaptive=False, max_rounds=None, y0=None, resync=False,
                 reuse=False):
    """The oracle's Alg. 1 for chain c next to a device trajectory tj [K+1, d] of a whole sample.

    Each round is the oracle's own (from its own state y[a]; from the device's state tj[a] if resync);
    on unflagged slots the oracle's decision stands, on a flagged slot of the walked prefix the branch is
    read off the device's row of that step (it equals one of the two branch values) and followed.
    reuse: model values carried across rounds on the oracle's side as well (a whole window accepted -- on the
    branch the device took -- hands the value at yhat_b to the next round).
    Returns dict(y, a, R, flips, flagged_slots, round_err, first_calls): y the oracle's trajectory up to a, R
    rounds, round_err the largest relative error of the rows written by a single round, first_calls the
    rounds that made a draft call of their own."""
    K, d = cfg["K"], cfg["d"]
    L = L or cfg["L"]
    xi, u = chain_randoms(seed, c, K, d)
    y = np.zeros((K + 1, d))
    y[0] = xi[0] if y0 is None else y0
    a = R = flips = nflag = first_calls = 0
    round_err = 0.0
    state = oasd.window_init(L)
    g_carry = None
    while a < K and (max_rounds is None or R < max_rounds):
        win = oasd.window_of(state, L) if adaptive else L
        start = np.asarray(tj[a], dtype=np.float64) if resync else y[a]
        rec = oasd.asd_round(start, a, win, T["c_x"], T["c_0"], T["sigma"], model, xi, u, eps=tol, g_a=g_carry,
                             evaluate_end=reuse)
        first_calls += rec["made_first_call"]
        w = rec["b"] - a
        n = 0
        while n < w:
            bit = bool(rec["acc"][n])
            if rec["flagged"][n]:
                nflag += 1
                row = np.asarray(tj[a + n + 1], dtype=np.float64)
                dev_bit = bool(np.max(np.abs(row - rec["yhat"][n])) <= np.max(np.abs(row - rec["z_rej"][n])))
                flips += dev_bit != bit
                bit = dev_bit
            if not bit:
                break
            n += 1
        y_new, a_next = outcome(rec, n)
        g_carry = rec["g_end"] if (reuse and n == w) else None
        round_err = max(round_err, rel_err(tj[a + 1: a_next + 1], y_new))
        y[a + 1: a_next + 1] = y_new
        state = oasd.window_next(state, w, n)
        a = a_next
        R += 1
    return dict(y=y, a=a, R=R, flips=flips, flagged_slots=nflag, round_err=round_err, first_calls=first_calls)
