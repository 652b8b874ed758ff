"""Puts a synthetic workload on the device and opens a library context for it.
Allocation and upload only (PyTorch as the memory manager)."""
import numpy as np
import torch

from . import binding


def device_params(cfg, params, device="cuda:0"):
    """Upload denoiser parameters (numpy, from asd_workloads) as device tensors.
    bf16 bit patterns travel as int16 tensors."""
    dev = torch.device(device)

    def up(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            a = a.view(np.int16)
        return torch.from_numpy(a).to(dev)

    if cfg["kind"] == "gmm":
        return dict(kind="gmm", d=cfg["d"], C=cfg["C"], var=params["var"], means=up(params["means"]),
                    log_w=up(params["log_w"]))
    out = dict(kind="mlp", d=cfg["d"], width=cfg["width"], n_blocks=cfg["n_blocks"], temb_dim=cfg["E"],
               out_clip=float(params.get("out_clip", 0.0)), predict_eps=bool(params.get("predict_eps", False)),
               act_terms=int(params.get("act_terms", 1)))
    for k in ("w_in", "w_blk", "w_out", "b_in", "b_blk", "b_out", "temb"):
        out[k] = up(params[k])
    return out


def open_ctx(cfg, params, seed=0, device="cuda:0", beta_min=1e-4, beta_max=0.02, L=None, chains=None):
    """Context for a workload dict (asd_workloads.CONFIGS entry) with the
    library's own linear-beta schedule (or, cfg["schedule"] == "cosine", its cosine one)."""
    if cfg.get("schedule", "linear") == "cosine":
        sched = binding.asd_schedule_from_abar(binding.asd_abar_cosine(cfg["K"]))
    else:
        sched = binding.asd_schedule_ddpm_linear(cfg["K"], beta_min, beta_max)
    den = device_params(cfg, params, device)
    den["n_tau"] = cfg["K"] + 1
    if cfg["kind"] == "gmm" or den.get("predict_eps"):
        den["abar"] = sched["abar"]
    ctx = binding.Ctx(sched, den, L or cfg["L"], chains or cfg["chains"], seed)
    ctx.sched = sched
    return ctx


def alloc_traj(ctx, device="cuda:0"):
    return torch.empty((ctx.chains, ctx.K + 1, ctx.d), dtype=torch.float32, device=device)
