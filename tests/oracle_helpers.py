"""Glue used by tests: oracle models and per-chain random inputs for a workload."""
import numpy as np

import asd_workloads as W
from oracle import denoisers, philox, schedule


def chain_randoms(seed, chain, K, d):
    """xi [K+1, d] (row 0 is the y_0 draw) and u [K+1] (index 0 unused)."""
    xi = philox.normals(seed, chain, range(K + 1), d)
    u = np.concatenate([[np.nan], philox.uniforms(seed, chain, range(1, K + 1))])
    return xi, u


def gmm_model(T, p):
    means = np.asarray(p["means"], dtype=np.float64)
    log_w = np.asarray(p["log_w"], dtype=np.float64)

    def model(idx, rows):
        tau = T["tau"][np.asarray(idx)]
        return denoisers.gmm_posterior_mean(rows, T["abar"][tau], means, log_w, p["var"])
    return model


def mlp_model(T, p):
    net = denoisers.MLPOracle(p, abar=T["abar"] if p.get("predict_eps") else None)

    def model(idx, rows):
        return net(rows, T["tau"][np.asarray(idx)])
    return model


def oracle_setup(cfg, model_seed=1):
    """(tables, params, model) of a workload dict from asd_workloads.CONFIGS."""
    if cfg.get("schedule", "linear") == "cosine":
        T = schedule.tables_from_abar(schedule.cosine_abar(cfg["K"]))
    else:
        T = schedule.ddpm_tables(cfg["K"], W.BETA_MIN, W.BETA_MAX)
    p = W.make_params(cfg, model_seed)
    model = gmm_model(T, p) if cfg["kind"] == "gmm" else mlp_model(T, p)
    return T, p, model
