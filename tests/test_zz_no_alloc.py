"""asd_sample_noalloc (the entry point for callers that cannot allocate) against asd_sample, through the C
boundary: same kernels with the verify call's outputs in the library's static scratch, so the samples must
agree (to the parity bar; in fact bit for bit).  Two calls in a row share the scratch, the second on a smaller
problem; a problem beyond the scratch is refused."""
import numpy as np
import pytest
import torch

import asd_workloads as W
from oracle_helpers import oracle_setup

pytestmark = pytest.mark.gpu

from paper_2505_03983_amd import binding, runtime   # noqa: E402
import gpu_helpers as H                              # noqa: E402

DEV = "cuda:0"


def _pair(cfg, p, seed, chains=None, L=None, adaptive=False, reuse=False):
    ctx = runtime.open_ctx(cfg, p, seed=seed, chains=chains, L=L)
    ctx.use_call_reuse(reuse)
    ctx.use_resident(False)          # asd_sample on the same lock-step round kernels, plainly launched
    ctx.use_graphs(False)
    ctx.use_adaptive_window(adaptive)
    ta, tb = runtime.alloc_traj(ctx), runtime.alloc_traj(ctx)
    ra = torch.zeros(ctx.chains, dtype=torch.int32, device=DEV)
    rb = torch.zeros_like(ra)
    na = ctx.sample(ta, ra)
    nb = ctx.sample_noalloc(tb, rb)
    torch.cuda.synchronize()
    tol = H.TOL[cfg["kind"]]
    e = H.rel_err(tb.cpu().numpy(), ta.cpu().numpy())
    print("no-alloc sample vs asd_sample:", cfg["kind"], "chains", ctx.chains, "L", ctx.L, "rel err", e,
          "bit-identical", bool(torch.equal(ta, tb)), "rounds", na, nb, flush=True)
    assert e <= tol
    assert torch.equal(ra, rb) and na == nb
    assert bool(torch.isfinite(tb).all().item())
    ctx.close()


def test_noalloc_sample_equals_sample_twice_in_a_row_second_smaller():
    cfg = W.CONFIGS[2]
    _, p, _ = oracle_setup(cfg)
    _pair(cfg, p, seed=7)                          # 64 chains, L = 16: 256 KB of scratch
    _pair(cfg, p, seed=8, chains=5, L=7)           # smaller: the scratch still holds the first call's values
    _pair(cfg, p, seed=9, chains=9, adaptive=True)
    _pair(cfg, p, seed=11, chains=7, reuse=True)   # L + 1 slots per chain in the scratch
    small_mlp = dict(kind="mlp", d=16, E=8, width=64, n_blocks=2, K=30, chains=6, L=12)
    _, pm, _ = oracle_setup(small_mlp)
    _pair(small_mlp, pm, seed=10)
    # a shape on which the early accept kernel and the rounds launched without the kernels behind it are at work
    # (17 k model rows per call; 8.5 MiB of scratch, which the chains left to the verify call use)
    early = dict(kind="gmm", d=128, C=256, K=200, chains=272, L=64, var=0.25)
    _, pe, _ = oracle_setup(early)
    _pair(early, pe, seed=12)


def test_noalloc_sample_refuses_what_does_not_fit_and_states_the_limit():
    cfg = dict(kind="gmm", d=64, C=4, K=4, chains=4096, L=64, var=0.25)     # 64 MiB of x0hat > 32 MiB
    _, p, _ = oracle_setup(cfg)
    ctx = runtime.open_ctx(cfg, p, seed=0)
    traj = runtime.alloc_traj(ctx)
    with pytest.raises(binding.AsdError) as ei:
        ctx.sample_noalloc(traj)
    assert ei.value.status == binding.ASD_EUNSUPPORTED and "static scratch" in str(ei.value)
    ctx.sample(traj)                               # the allocating entry point serves it
    assert bool(torch.isfinite(traj).all().item())
    ctx.close()
    cfg2 = W.CONFIGS[1]
    _, p2, _ = oracle_setup(cfg2)
    ctx2 = runtime.open_ctx(cfg2, p2, seed=0)
    ctx2.profile_enable(True)
    with pytest.raises(binding.AsdError) as ei:
        ctx2.sample_noalloc(runtime.alloc_traj(ctx2))
    assert ei.value.status == binding.ASD_ESTATE
    ctx2.close()
