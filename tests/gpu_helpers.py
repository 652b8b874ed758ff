"""Helpers of the GPU parity tests: run the library on oracle-chosen states."""
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


def rel_err(got, want):
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    if want.size == 0:
        return 0.0
    return float(np.max(np.abs(got - want)) / max(1.0, np.max(np.abs(want))))


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


def compare_round(out, c, rec, tol, K, x0_scale=1.0):
    """Compare device results of chain c with the oracle's record of the same round.
    Returns (ok_bits, first_flagged) and asserts on everything else."""
    a, b = rec["a"], rec["b"]
    w = b - a
    # proposal samples
    e = rel_err(out["drafted"][c][a + 1: b + 1], rec["yhat"])
    assert e <= tol, ("yhat", c, a, e)
    # model values at slots 0..w-1
    # For the clipped bf16 network the rounding noise lives on the scale of the *unclipped* output
    # (x0_scale = max |unclipped oracle output| over these rows, >= 1), which the clip then hides.
    e = rel_err(out["x0hat"][c][:w], rec["g"]) / max(1.0, x0_scale)
    assert e <= tol, ("x0hat", c, a, e)
    # decisions: exact off flagged near-ties, walking the prefix as Alg. 2 does
    n_acc_dev = int(out["accepted"][c])
    n_acc = rec["j"] - a
    prefix_flag = rec["flagged"][: min(n_acc + 1, w)].any()
    if not prefix_flag:
        assert n_acc_dev == n_acc, ("prefix", c, a, n_acc_dev, n_acc)
    if n_acc_dev != n_acc:
        return False
    assert out["a_next"][c] == rec["a_next"]
    # values written by the round
    e = rel_err(out["traj"][c][a + 1: rec["a_next"] + 1], rec["y_new"])
    assert e <= tol, ("y_new", c, a, e)
    return True
