"""Seeded synthetic inputs for the five ASD workloads.

Shared by the tests, the benchmark and the CPU oracle.  It holds no
arithmetic of the sampling method: only the shapes of the workloads and the
seeded draws of denoiser parameters (mixture means, MLP weights, the
sinusoidal time-embedding table), which both sides consume as data.

The workloads stand in for the paper's experiments (Sec. 5): the
diffusion-policy shape (16 x 7 actions, K = 100, batched verification on one
GPU) and image-shaped models at K = 1000, whose trained weights are not
available; Gaussian-mixture data gives a denoiser with a closed form.
"""
import numpy as np

BETA_MIN = 1e-4
BETA_MAX = 0.02

CONFIGS = {
    1: dict(kind="gmm", d=2, C=4, K=100, chains=8, L=8, var=0.25),
    2: dict(kind="gmm", d=64, C=256, K=1000, chains=64, L=16, var=0.25),
    3: dict(kind="mlp", d=112, E=128, width=1024, n_blocks=4, K=100, chains=256, L=16),
    4: dict(kind="mlp", d=3072, E=256, width=4096, n_blocks=6, K=1000, chains=64, L=32),
    5: dict(kind="gmm", d=1024, C=4096, K=1000, chains=1024, L=64, var=0.25),
}


def _rng(seed, stream):
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def gmm_params(d, C, var=0.25, model_seed=1):
    """Means ~ N(0, 4 I) (std 2 per coordinate), uniform weights; fp32."""
    rng = _rng(model_seed, 1)
    means = (2.0 * rng.standard_normal((C, d))).astype(np.float32)
    log_w = np.full(C, -np.log(C), dtype=np.float32)
    return dict(means=means, log_w=log_w, var=float(var))


def f32_to_bf16_bits(a):
    """fp32 -> bf16 bit patterns (uint16), round to nearest even, via torch."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def sinusoidal_table(n_rows, E):
    """Row tau: [sin(tau w_k), cos(tau w_k)], w_k = 10000^(-k/(E/2)), bf16 bits."""
    half = E // 2
    k = np.arange(half, dtype=np.float64)
    w = 10000.0 ** (-k / half)
    ang = np.arange(n_rows, dtype=np.float64)[:, None] * w[None, :]
    tab = np.concatenate([np.sin(ang), np.cos(ang)], axis=1)
    return f32_to_bf16_bits(tab.astype(np.float32))


def mlp_params(d, E, width, n_blocks, K, model_seed=1, out_clip=1.0, predict_eps=False, act_terms=2):
    """Weights ~ N(0, 1/fan_in) rounded to bf16 (uint16 patterns), zero biases
    (fp32), time-embedding table [K+1, E] (bf16 patterns), row-major [out, in].
    out_clip: the predicted x_0 is clipped to [-1, 1] as DDPM samplers commonly
    do (a random-weight network is not a contraction; without the clip the
    chain leaves the fp32 range within a few hundred steps).
    act_terms: bf16 terms an fp32 activation enters a matrix product with (a setting of the
    denoiser, passed through to both sides)."""
    rng = _rng(model_seed, 2)

    def w(out_f, in_f):
        a = rng.standard_normal((out_f, in_f), dtype=np.float32) / np.float32(np.sqrt(in_f))
        return f32_to_bf16_bits(a)

    return dict(
        w_in=w(width, d + E),
        w_blk=np.stack([w(width, width) for _ in range(n_blocks)]),
        w_out=w(d, width),
        b_in=np.zeros(width, dtype=np.float32),
        b_blk=np.zeros((n_blocks, width), dtype=np.float32),
        b_out=np.zeros(d, dtype=np.float32),
        temb=sinusoidal_table(K + 1, E),
        out_clip=float(out_clip),
        predict_eps=bool(predict_eps),
        act_terms=int(act_terms),
    )


def make_params(cfg, model_seed=1):
    if cfg["kind"] == "gmm":
        return gmm_params(cfg["d"], cfg["C"], cfg["var"], model_seed)
    return mlp_params(cfg["d"], cfg["E"], cfg["width"], cfg["n_blocks"], cfg["K"], model_seed,
                      predict_eps=cfg.get("predict_eps", False), act_terms=cfg.get("act_terms", 2))
