#!/usr/bin/env python3
"""Benchmark of the ASD hot path on one MI355X.

One "step" of this benchmark is one complete `asd_sample` over the whole batch
of chains of the workload: every round (draft model call, draft, batched
verify model call, accept/scan/resample) until every chain has reached K.
The metric is DDPM steps per second = chains * K / wall-clock of a sample,
with all inputs resident in HBM before the timed region starts.

Prints ONE JSON line.  Besides the
throughput it carries
  roofline      the dominant kernel of the workload against the MI355X peak,
                timed live with HIP events on the launch stream,
  cpu_baseline  the CPU oracle timed on this machine's host cores on a
                bounded sample of the same workload (a reported baseline).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

PEAK = {"f32": 157.3, "bf16": 2500.0, "f16": 2500.0, "i8": 5000.0}          # dense MFMA TFLOP/s (int8: TOP/s), MI355X
HBM_PEAK_GBS = 8000.0

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "cfg5_gmm_verify_gemm_hbm_traffic.txt")


def traffic_bytes_per_launch(w, kernel, arithmetic):
    """HBM-side bytes per launch of a verify GEMM as rocprofv3 measured them (FETCH_SIZE and WRITE_SIZE, each
    scaled by what the same counter reads for a plain copy of known size): parsed from the committed summary
    of those runs, whose `TRAFFIC` lines carry the readings and the scale factors.  None if it has no line
    for this kernel."""
    import re
    try:
        text = open(TRAFFIC_FILE).read()
    except OSError:
        return None
    for line in text.splitlines():
        if not line.startswith("TRAFFIC "):
            continue
        kv = dict(re.findall(r"(\w+)=(\S+)", line))
        if kv.get("workload") == str(w) and kv.get("kernel") == kernel and kv.get("arithmetic") == arithmetic:
            return 1024.0 * (float(kv["fetch_scale"]) * float(kv["fetch_kib"]) +
                             float(kv["write_scale"]) * float(kv["write_kib"]))
    return None


def workload_name(w, cfg):
    if cfg["kind"] == "gmm":
        return "cfg%d: GMM denoiser d=%d C=%d K=%d chains=%d L=%d fp32" % (
            w, cfg["d"], cfg["C"], cfg["K"], cfg["chains"], cfg["L"])
    return "cfg%d: MLP denoiser d=%d E=%d width=%d blocks=%d K=%d chains=%d L=%d bf16 weights, fp32 state" % (
        w, cfg["d"], cfg["E"], cfg["width"], cfg["n_blocks"], cfg["K"], cfg["chains"], cfg["L"])


class ClockSampler:
    """Shader clock of GPU 0 as rocm-smi reports it, polled from a host thread while a region runs (a child
    process per poll; nothing is launched on the GPU).  The chip lowers it under dense matrix work."""

    def __init__(self, period_s=0.2):
        import threading
        self.period, self.samples, self._stop = period_s, [], threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True)

    def _run(self):
        import re
        import subprocess
        while not self._stop.is_set():
            try:
                out = subprocess.run(["/opt/rocm/bin/rocm-smi", "-d", "0", "--showclocks"], capture_output=True,
                                     text=True, timeout=5).stdout
                m = re.search(r"sclk clock level: \d+: \((\d+)Mhz\)", out)
                if m:
                    self.samples.append(int(m.group(1)))
            except Exception:
                return
            self._stop.wait(self.period)

    def __enter__(self):
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        self._thread.join(timeout=10)

    def summary(self):
        if not self.samples:
            return None
        return dict(samples=len(self.samples), min=min(self.samples), max=max(self.samples),
                    mean=sum(self.samples) / len(self.samples), last=self.samples[-1])


def run_gpu(w, steps, warmup, seed, profile=True, adaptive=False, split=True, clocks=False, act_terms=None,
            screen=None):
    import torch
    import asd_workloads as W
    from paper_2505_03983_amd import binding, runtime

    cfg = W.CONFIGS[w]
    if act_terms is not None and cfg["kind"] == "mlp":
        cfg = dict(cfg, act_terms=act_terms)
    params = W.make_params(cfg, model_seed=1)
    ctx = runtime.open_ctx(cfg, params, seed=seed)
    ctx.use_adaptive_window(adaptive)
    ctx.use_split_gemm(split)
    split_active = ctx.split_gemm_active()
    split_products = ctx.split_gemm_products()
    if screen is not None:
        ctx.use_logit_screen(screen)
    screen_mode = ctx.logit_screen_active()
    traj = runtime.alloc_traj(ctx)
    rounds = torch.zeros(cfg["chains"], dtype=torch.int32, device="cuda:0")
    for i in range(warmup):
        ctx.set_seed(seed + 1000 + i)
        ctx.sample(traj, rounds)
    torch.cuda.synchronize()
    if profile:
        # profile = True: every kernel of the path is bracketed by events; a list: those slots only (an event ends
        # the overlap of the kernels around it and costs a few microseconds: two thousand of them per sample of
        # workload 5 are a tenth of its time, the four per round around the two verify GEMMs are not)
        ctx.profile_select(None if profile is True else profile)
        ctx.profile_enable(True)
    path = "chain-resident kernel, one launch per sample" if ctx.resident_active() else \
        "lock-step round kernels" + ((", plain launches, events around every kernel" if profile is True else
                                      ", plain launches, events around " + " and ".join(profile)) if profile
                                     else ", one captured graph per round")
    launched = []
    rmean, rmax = [], []
    sampler = ClockSampler() if clocks else None
    if sampler:
        sampler.__enter__()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        ctx.set_seed(seed + i)
        launched.append(ctx.sample(traj, rounds))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if sampler:
        sampler.__exit__()
    r = rounds.cpu().numpy()
    rmean.append(float(r.mean()))
    rmax.append(int(r.max()))
    finite = bool(torch.isfinite(traj[:, -1]).all().item())
    wall = t1 - t0
    out = dict(cfg=cfg, wall_s=wall, steps_per_s=cfg["chains"] * cfg["K"] * steps / wall,
               ms_per_sample=1e3 * wall / steps, rounds_mean=rmean[-1], rounds_max=rmax[-1],
               rounds_launched=launched, finite=finite, path=path, split=split_active, split_products=split_products,
               act_terms=params.get("act_terms"), sclk_mhz=sampler.summary() if sampler else None,
               screen_mode=screen_mode)
    if profile:
        P = binding.PROF
        table = {}
        for name, kid in P.items():
            for call in (0, 1):
                n, ms = ctx.profile_read(kid, call)
                if n:
                    table["%s/%s" % (name, "verify" if call else "draft")] = dict(launches=n, total_ms=ms,
                                                                                 avg_us=1e3 * ms / n)
        out["kernels"] = table
        out["rows"] = ctx.profile_rows()
        out["accept_rows"] = ctx.profile_accept_rows()
        out["early_accept"] = ctx.profile_early_accept() if ctx.early_accept_active() else None
        out["model_work"] = ctx.profile_model_work()
        ctx.profile_enable(False)
        ctx.profile_select(None)
    ctx.close()
    del traj
    torch.cuda.empty_cache()
    return out


def roofline(res, w=None, kernel=None):
    """Roofline entry of the dominant kernel of a profiled run.

    Mixture denoiser: one GEMM of the model call does 2*C*d flop per row (the method's arithmetic, fp32).  The
    default kernels evaluate every fp32 product as three fp16 MFMA products (two fp16 terms per operand; six bf16
    products of three terms where d or C is not a multiple of 32), so they *execute* three (six) times that on
    the 16-bit pipe.  `achieved` / `peak` / `frac` are the executed 16-bit work against that pipe's MFMA peak (how
    busy the pipe in use is); `method` carries the 2*C*d figure and its ratio to the fp32 MFMA peak.
    Both split-operand GEMMs leave out work whose result is known to be exact zeros (tiles of logits far below
    their rows' maxima, found by the screening pass; slabs of components with zero weights): what they executed
    is then counted by the device (half tiles of 64 rows x 128 components, slabs of 32 or 16 components per tile) and
    not inferred from rows."""
    cfg, k = res["cfg"], res["kernels"]
    draft_rows, verify_rows = res["rows"]
    executed_per_method = 1.0
    executed_flops = None
    if cfg["kind"] == "gmm":
        cand = [n for n in ("GMM_LOGITS/verify", "GMM_COMBINE/verify", "GMM_ROWWISE/verify") if n in k]
        name = kernel or max(cand, key=lambda n: k[n]["total_ms"])      # the one the sample spends most time in
        launches = k[name]["launches"]
        # 2*C*d flops per row for either GEMM (the row-wise kernel does both: 4*C*d)
        per_row = (4.0 if name.startswith("GMM_ROWWISE") else 2.0) * cfg["C"] * cfg["d"]
        dtype = "f32"
        # the row-wise kernel runs on the vector ALUs; its bound is the fp32 vector peak (same figure)
        bound = "mfma" if not name.startswith("GMM_ROWWISE") else "alu"
        if bound == "mfma" and res.get("split"):
            executed_per_method = float(res.get("split_products") or 6)
            dtype = "f16" if executed_per_method == 3.0 else "bf16"
            slab = 32 if executed_per_method == 3.0 else 16                      # components per K slab of the second GEMM
            done, tiles, slabs_done, slabs = res.get("model_work", (0, 0, 0, 0, 0, 0, 0))[:4]
            if name == "GMM_LOGITS/verify" and tiles:
                executed_flops = executed_per_method * 2.0 * 64 * 128 * cfg["d"] * done / launches   # half tiles of 64 rows
            if name == "GMM_COMBINE/verify" and slabs:
                executed_flops = executed_per_method * 2.0 * 128 * 128 * slab * slabs_done / launches
    else:
        name = "MLP_GEMM_BLK/verify"
        launches = k[name]["launches"]
        per_row = 2.0 * cfg["width"] * cfg["width"]
        verify_rows = verify_rows * cfg["n_blocks"]      # one launch per block, each over all rows
        dtype = "bf16"
        bound = "mfma"
        executed_per_method = float(res.get("act_terms", 1))   # each activation term is multiplied with the weights
    method_flops = per_row * verify_rows / launches
    avg_s = 1e-3 * k[name]["total_ms"] / launches
    method_tflops = method_flops / avg_s / 1e12
    if executed_flops is None:
        executed_flops = executed_per_method * method_flops
    achieved = executed_flops / avg_s / 1e12
    peak = PEAK[dtype]
    out = dict(bound=bound, kernel=name, achieved=achieved, peak=peak, unit="TFLOP/s", frac=achieved / peak,
               frac_is="executed %s MFMA flop/s over the %s MFMA peak" % (dtype, dtype) if bound == "mfma"
               else "executed fp32 flop/s over the fp32 vector peak",
               traffic=traffic_bytes_per_launch(w, name, dtype), avg_launch_us=1e6 * avg_s, launches=launches,
               executed_flops_per_launch=executed_flops, mfma_dtype=dtype,
               share_of_wall=1e-3 * k[name]["total_ms"] / res["wall_s"])
    if cfg["kind"] == "gmm":
        out["method"] = dict(flops_per_launch=method_flops, what="2*C*d per row (fp32 contraction of the model call)",
                             tflops=method_tflops, fp32_mfma_peak=PEAK["f32"],
                             ratio_to_fp32_mfma_peak=method_tflops / PEAK["f32"])
        out["executed_16bit_products_per_fp32_product"] = int(executed_per_method)
        if executed_flops != executed_per_method * method_flops:
            out["executed_share_of_dense"] = executed_flops / (executed_per_method * method_flops)
    else:
        out["method"] = dict(flops_per_launch=method_flops, what="2*width^2 per row and block",
                             tflops=method_tflops, bf16_terms_per_activation=int(executed_per_method))
    return out


def logit_screen(res):
    """The int8 screening pass of the mixture denoiser's verify calls: its cost, what it saved, and how busy it keeps
    the int8 matrix pipe (2 * 64 * 128 * d operations per screened half tile against the 5 POP/s data-sheet peak)."""
    k = res["kernels"]
    if not res.get("screen_mode") or "GMM_SCREEN/verify" not in k:
        return dict(mode=res.get("screen_mode", 0))
    done, tiles, _, _, screened, onehot, certified = res["model_work"]
    s = k["GMM_SCREEN/verify"]
    ops = 2.0 * 64 * 128 * res["cfg"]["d"] * screened
    return dict(mode=res["screen_mode"], launches=s["launches"], total_ms=s["total_ms"],
                share_of_wall=1e-3 * s["total_ms"] / res["wall_s"],
                logit_half_tiles=tiles, logit_half_tiles_of_screened_calls=screened, logit_half_tiles_computed=done,
                computed_share=done / tiles if tiles else None,
                row_tiles_of_second_gemm_in_closed_form=onehot, row_tiles_certified_before_any_matrix_work=certified,
                certificate=({"launches": k["GMM_CERT/verify"]["launches"], "total_ms": k["GMM_CERT/verify"]["total_ms"],
                              "share_of_wall": 1e-3 * k["GMM_CERT/verify"]["total_ms"] / res["wall_s"],
                              "note": "one kernel: reads a row, tests it, writes its result if it passes"}
                             if "GMM_CERT/verify" in k else None),
                int8_tops=ops / (1e-3 * s["total_ms"]) / 1e12 if screened else 0.0, int8_peak_tops=PEAK["i8"],
                note="total_ms covers the quantiser, the int8 GEMM and the decision kernel; calls the draft call's "
                     "verdict switched the screen off for still launch all three (they exit at once)")


def hbm_kernels(res):
    """Algorithmic HBM bytes per second of the draft and accept kernels (event-timed: a few microseconds of
    launch overhead are inside each figure; profiles/ has the rocprofv3 durations).  Both kernels regenerate
    their noise (Philox4x32-10 + Box-Muller per four coordinates) and are bound by that arithmetic, not by HBM;
    the figures say how far from the HBM roof that leaves them.
    draft: reads y_a and x0a (2 rows per live chain), writes the w drafted rows.
    accept: reads x0a and the x0hat rows of the slots it examines -- it walks the window eight slots at a time
    and stops at the group holding the first rejection, so it reads far fewer than the w - 1 rows of the window
    (the count comes from the device) -- and, on a rejection, reads and rewrites one trajectory row.
    `whole_window` is the same figure had it read every slot: an upper bound, kept for comparison."""
    cfg, k = res["cfg"], res["kernels"]
    draft_rows, verify_rows = res["rows"]
    examined, resampled = res.get("accept_rows", (None, None))
    d = cfg["d"]
    w_total = verify_rows + draft_rows      # w summed over chains and rounds
    chain_rounds = draft_rows               # one draft-call row per live chain and round
    ea = res.get("early_accept")
    if ea:
        # chain-rounds the early accept kernel took whole: neither the draft kernel nor the accept kernel saw them
        e_rows, e_rounds, e_window, e_resampled = ea
        w_total -= e_window + e_rounds
        chain_rounds -= e_rounds
        if examined is not None:
            examined, resampled = examined - e_rows, resampled - e_resampled
        verify_rows -= e_window
    out = {}
    if "DRAFT/draft" in k:
        b = 4.0 * d * (2 * chain_rounds + w_total)
        out["draft"] = dict(GBps=b / (1e-3 * k["DRAFT/draft"]["total_ms"]) / 1e9,
                            avg_us=k["DRAFT/draft"]["avg_us"], bytes_per_launch=b / k["DRAFT/draft"]["launches"])
    if "ACCEPT/draft" in k:
        t = 1e-3 * k["ACCEPT/draft"]["total_ms"]
        whole = 4.0 * d * (w_total + 3 * chain_rounds)
        out["accept"] = dict(avg_us=k["ACCEPT/draft"]["avg_us"],
                             whole_window=dict(GBps=whole / t / 1e9, frac_of_hbm_peak=whole / t / 1e9 / HBM_PEAK_GBS))
        if examined is not None:
            b = 4.0 * d * (examined + chain_rounds + 2 * resampled)
            out["accept"].update(GBps=b / t / 1e9, bytes_per_launch=b / k["ACCEPT/draft"]["launches"],
                                 share_of_window_rows_read=examined / max(1.0, float(verify_rows)))
        else:
            out["accept"]["GBps"] = whole / t / 1e9
    if ea and "ACCEPT_EARLY/draft" in k:
        # reads y_a, x0a and mu_b per chain-round; writes the rows the chain keeps (about the examined ones)
        t = 1e-3 * k["ACCEPT_EARLY/draft"]["total_ms"]
        b = 4.0 * d * (3 * ea[1] + ea[0])
        out["accept_early"] = dict(GBps=b / t / 1e9, avg_us=k["ACCEPT_EARLY/draft"]["avg_us"],
                                   bytes_per_launch=b / k["ACCEPT_EARLY/draft"]["launches"],
                                   chain_rounds_taken=ea[1], share_of_chain_rounds=ea[1] / max(1.0, float(draft_rows)),
                                   model_rows_formed=ea[0], window_rows_spared_the_verify_call=ea[2])
    for v in out.values():
        v["frac_of_hbm_peak"] = v["GBps"] / HBM_PEAK_GBS
        v["bound_by"] = "ALU (counter-based noise regenerated in registers)"
    return out


def cpu_baseline(w, seed, budget_s=24.0, n_phases=8):
    """The oracle as it stands, timed on the host on one thread.

    A round of Alg. 1 advances many steps while the noise is large and few near the end, so a rate taken
    from the first rounds of a chain overstates the oracle.  Whole chains are timed when one fits in the
    budget (workloads 1-3).  Otherwise the chain is sampled at n_phases phases (a = 0, K/n, 2K/n, ...): from
    a synthetic state of that noise level -- a draw from the forward marginal of the data law, which is the law
    of y_a since the chain is exact -- the oracle runs rounds for its share of the budget, and the chain's rate
    is the steps-weighted harmonic mean of the phase rates (each phase stands for K/n steps; most of a chain's
    time goes to its last phases, where a round advances few steps)."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import asd_workloads as W
    from oracle import asd as oasd
    from oracle_helpers import chain_randoms, oracle_setup
    try:
        from threadpoolctl import threadpool_limits
    except Exception:                                   # pragma: no cover
        threadpool_limits = None
    cfg = W.CONFIGS[w]
    T, p, model = oracle_setup(cfg)
    K, L, d = cfg["K"], cfg["L"], cfg["d"]
    ctxmgr = threadpool_limits(limits=1) if threadpool_limits else None
    host_cores = os.cpu_count()

    def run_rounds(y, a, xi, u, t_end, stop_at=K):
        steps = rounds = 0
        while a < stop_at and time.perf_counter() < t_end:
            rec = oasd.asd_round(y, a, L, T["c_x"], T["c_0"], T["sigma"], model, xi, u)
            y = rec["y_new"][-1]
            steps += rec["a_next"] - a
            a = rec["a_next"]
            rounds += 1
        return steps, rounds, a

    try:
        t0 = time.perf_counter()
        xi, u = chain_randoms(seed, 0, K, d)
        s1, r1, a1 = run_rounds(xi[0], 0, xi, u, t0 + 1e-9)          # one round, to size the job
        t_round = time.perf_counter() - t0
        whole = t_round * (K / max(1, s1)) * 3.0 < 0.5 * budget_s        # late rounds advance ~3x less
        if whole:
            steps = rounds = chains = 0
            t0 = time.perf_counter()
            while time.perf_counter() - t0 < budget_s:
                xi, u = chain_randoms(seed, chains, K, d)
                s_, r_, a_ = run_rounds(xi[0], 0, xi, u, float("inf"))
                steps, rounds, chains = steps + s_, rounds + r_, chains + 1
            el = time.perf_counter() - t0
            value = steps / el
            sample = ("%d whole chains (chain ids 0..%d: %d ASD rounds, %d DDPM steps) of the same workload, %.1f s"
                      % (chains, chains - 1, rounds, steps, el))
        else:
            rng = np.random.default_rng(seed)
            phases, inv = [], 0.0
            t_all = time.perf_counter()
            for ph in range(n_phases):
                a0 = ph * K // n_phases
                xi, u = chain_randoms(seed, ph, K, d)
                if a0 == 0:
                    y = xi[0]
                else:
                    ab = T["abar"][T["tau"][a0]]
                    if cfg["kind"] == "gmm":
                        x0 = p["means"][rng.integers(0, cfg["C"])] + np.sqrt(p["var"]) * rng.standard_normal(d)
                    else:
                        x0 = rng.uniform(-1.0, 1.0, d)
                    y = np.sqrt(ab) * x0 + np.sqrt(1.0 - ab) * rng.standard_normal(d)
                t0 = time.perf_counter()
                s_, r_, a_ = run_rounds(y, a0, xi, u, t0 + budget_s / n_phases)
                el = time.perf_counter() - t0
                phases.append(dict(a=a0, rounds=r_, steps=s_, seconds=round(el, 2), steps_per_s=s_ / el))
                inv += (1.0 / n_phases) / (s_ / el)
            value = 1.0 / inv
            sample = ("rounds of single chains from %d phases of the chain (a = 0, K/%d, ...; synthetic states of that "
                      "noise level), an equal share of the budget each, combined as the steps-weighted harmonic mean: "
                      % (n_phases, n_phases)
                      + "; ".join("a=%d: %d rounds, %d steps, %.1f steps/s" % (q["a"], q["rounds"], q["steps"],
                                                                               q["steps_per_s"]) for q in phases)
                      + "; %.1f s in all" % (time.perf_counter() - t_all))
    finally:
        if ctxmgr is not None:
            ctxmgr.__exit__(None, None, None)
    return dict(value=value, unit="DDPM steps/s", cores=1, kind="oracle", host_cores_available=host_cores,
                sample=sample + "; fp64 numpy, one thread (BLAS limited to 1: the oracle's time is in element-wise "
                                "fp64 work, which numpy does not thread)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", type=int, default=5, help="1..5 (asd_workloads.CONFIGS)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--others", type=int, default=1, help="also time the other four workloads (1 sample each)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--plain", action="store_true",
                    help="time the sample without the library's per-kernel events (the production path: captured "
                         "graphs or the chain-resident kernel); the line then has no roofline object -- meant for "
                         "runs under rocprofv3, which times the kernels itself")
    ap.add_argument("--fp32-mfma", action="store_true",
                    help="Gaussian-mixture verify GEMMs on the fp32 matrix pipe instead of the 16-bit pipe with "
                         "split operands")
    ap.add_argument("--no-screen", action="store_true",
                    help="Gaussian-mixture verify calls without the int8 screening pass (every tile of logits computed)")
    ap.add_argument("--window-control", action="store_true",
                    help="time the sample with the per-chain window controller on (an extension of Alg. 1; the "
                         "default run keeps the configured fixed L and reports this mode in `window_control`)")
    ap.add_argument("--act-terms", type=int, default=None, choices=(1, 2),
                    help="MLP workloads: bf16 terms per activation (default: the workload's own setting, 2)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (a kernel of known HBM traffic, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (chains are independent, so a batch shards across GPUs by chain); "
              "got --gpus %d" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library is the only path (no CPU fallback)", file=sys.stderr)
        sys.exit(3)
    import asd_workloads as W

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                       # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    # (the clock is polled through rocm-smi child processes; under a profiler, whose preloaded library has
    # initialised the GPU in this process, such children may not be started, and --plain is the profiler mode)
    # The timed region carries events around the kernels the roofline object may be about (the exact GEMMs of the
    # verify call; the block GEMM of the network); a second, shorter pass with events around every kernel gives the
    # per-kernel table and the figures of the other kernels (all_kernel_events).
    kind = W.CONFIGS[args.workload]["kind"]
    cand = ["GMM_LOGITS/verify", "GMM_COMBINE/verify", "GMM_ROWWISE/verify"] if kind == "gmm" else ["MLP_GEMM_BLK/verify"]
    common = dict(split=not args.fp32_mfma, adaptive=args.window_control, act_terms=args.act_terms,
                  screen=0 if args.no_screen else None)
    res = run_gpu(args.workload, args.steps, args.warmup, args.seed, profile=False if args.plain else cand,
                  clocks=not args.plain, **common)
    if not res["finite"]:
        print("bench.py: non-finite samples", file=sys.stderr)
        sys.exit(4)
    cfg = res["cfg"]
    line = {
        "metric": "DDPM steps/s (chains*K/wall) for ASD at 1 GPU" + (" [window control on]" if args.window_control else ""),
        "value": res["steps_per_s"],
        "unit": "DDPM steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["ms_per_sample"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if cfg["kind"] == "gmm" else "bf16",
        "data": "synthetic",
        "config": {"workload": workload_name(args.workload, cfg), "chains": cfg["chains"], "K": cfg["K"],
                   "L": cfg["L"], "d": cfg["d"]},
        "rounds_per_sample": {"mean": res["rounds_mean"], "max": res["rounds_max"],
                              "launched": res["rounds_launched"]},
        "path": res["path"],
        "sclk_mhz_during_timed_region": res["sclk_mhz"],     # rocm-smi, polled from the host (nominal 2400)
    }
    if cfg["kind"] == "gmm":
        line["verify_gemm_arithmetic"] = (
            "fp32 MFMA" if not res["split"] else
            "every fp32 product as three fp16 MFMA products of two-term split operands, fp32 accumulation"
            if res["split_products"] == 3 else
            "every fp32 product as six bf16 MFMA products of three-way split operands, fp32 accumulation")
    else:
        line["mlp_activation_terms"] = res["act_terms"]
    if not args.plain:
        line["roofline"] = roofline(res, args.workload)
        if res["sclk_mhz"] and line["roofline"]["bound"] == "mfma":
            # the data-sheet peak is quoted at 2400 MHz; under dense matrix work the chip runs slower than that
            rf0 = line["roofline"]
            rf0["peak_at_measured_clock"] = rf0["peak"] * res["sclk_mhz"]["mean"] / 2400.0
            rf0["frac_at_measured_clock"] = rf0["achieved"] / rf0["peak_at_measured_clock"]
        rall = res      # (--others 0, the mode of the profiler runs: no second pass, the table has the GEMMs only)
        if args.others:
            rall = run_gpu(args.workload, max(1, min(args.steps, 5)), 1, args.seed, profile=True, **common)
            line["all_kernel_events"] = dict(steps_per_s=rall["steps_per_s"], ms_per_sample=rall["ms_per_sample"],
                                             samples=max(1, min(args.steps, 5)), path=rall["path"],
                                             note="the pass behind `kernels`, `hbm_kernels` and `logit_screen`")
        line["hbm_kernels"] = hbm_kernels(rall)
        if cfg["kind"] == "gmm" and res["split"]:
            line["logit_screen"] = logit_screen(rall)
            # the other exact GEMM of the verify call, by the same accounting
            other = [n for n in ("GMM_LOGITS/verify", "GMM_COMBINE/verify")
                     if n in res["kernels"] and n != line["roofline"]["kernel"]]
            line["roofline_other_verify_gemm"] = {
                n: {kk: vv for kk, vv in roofline(res, args.workload, kernel=n).items()
                    if kk in ("achieved", "peak", "frac", "avg_launch_us", "launches", "share_of_wall", "traffic",
                              "executed_flops_per_launch", "executed_share_of_dense")} for n in other}
        line["kernels"] = {k: {"launches": v["launches"], "avg_us": round(v["avg_us"], 2),
                               "total_ms": round(v["total_ms"], 3)} for k, v in rall["kernels"].items()}
    if not args.plain and args.others:
        # (skipped with --others 0, so that a profiler run of this script sees the sampling kernels only)
        # what the matrix pipes of this chip sustain on random operands with no memory traffic at all (the chip is
        # power-limited on dense MFMA work: the data-sheet peaks above hold for constant operands only)
        from paper_2505_03983_amd import probe
        sus = {"bf16": probe.asd_probe_mfma_ceiling(1, True, 300), "f16": probe.asd_probe_mfma_ceiling(2, True, 300),
               "f32": probe.asd_probe_mfma_ceiling(0, True, 300)}
        rf = line["roofline"]
        if rf["bound"] == "mfma":
            rf["sustained_random_operands"] = sus[rf["mfma_dtype"]]
            rf["frac_of_sustained"] = rf["achieved"] / sus[rf["mfma_dtype"]]
        line["mfma_sustained_random_operands_tflops"] = sus
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(args.workload, args.seed)
    # The same workload with the window controller on (windows <= L chosen per chain from its past:
    # an extension of Alg. 1, exact in law; the headline `value` above keeps the configured fixed L).
    # (Skipped with --others 0, so that a profiler run of this script sees the fixed-L launches only.)
    if args.others and not args.plain:
        # the same sample as the library runs it in production: no events, one captured graph per round
        # (or the chain-resident kernel); `value` above is the event-timed pass that the roofline figures come from
        rq = run_gpu(args.workload, max(1, min(args.steps, 5)), 1, args.seed, profile=False, **common)
        line["without_kernel_events"] = dict(steps_per_s=rq["steps_per_s"], ms_per_sample=rq["ms_per_sample"], path=rq["path"])
    if args.others and res["split"] and res["screen_mode"]:
        # the same sample with every tile of logits computed (asd_use_logit_screen off)
        rn = run_gpu(args.workload, 1, 1, args.seed, profile=cand, screen=0)
        rfn = roofline(rn, args.workload)
        line["unscreened"] = dict(steps_per_s=rn["steps_per_s"], ms_per_sample=rn["ms_per_sample"],
                                  roofline_kernel=rfn["kernel"], achieved=rfn["achieved"], frac=rfn["frac"],
                                  avg_launch_us=rfn["avg_launch_us"], share_of_wall=rfn["share_of_wall"])
    if args.others and res["split"]:
        # the same sample with the verify GEMMs on the fp32 matrix pipe (asd_use_split_gemm off)
        rp = run_gpu(args.workload, 1, 1, args.seed, profile=cand, split=False, clocks=True)
        rfp = roofline(rp, args.workload)
        line["fp32_mfma_path"] = dict(steps_per_s=rp["steps_per_s"], ms_per_sample=rp["ms_per_sample"],
                                      roofline_kernel=rfp["kernel"], achieved=rfp["achieved"], peak=rfp["peak"],
                                      frac=rfp["frac"], avg_launch_us=rfp["avg_launch_us"], traffic=rfp["traffic"],
                                      sclk_mhz_during_timed_region=rp["sclk_mhz"])
    if args.others:
        ra = run_gpu(args.workload, max(1, min(args.steps, 2)), 1, args.seed, profile=False, adaptive=True)
        line["window_control"] = dict(steps_per_s=ra["steps_per_s"], ms_per_sample=ra["ms_per_sample"],
                                      rounds_mean=ra["rounds_mean"], rounds_max=ra["rounds_max"], path=ra["path"])
    if args.others:
        others = {}
        for w in sorted(W.CONFIGS):
            if w == args.workload:
                continue
            r0 = run_gpu(w, 2, 1, args.seed, profile=False)      # throughput without the event overhead
            r = run_gpu(w, 1, 0, args.seed, profile=True)        # per-kernel figures
            ra = run_gpu(w, 2, 1, args.seed, profile=False, adaptive=True)
            rf = roofline(r)
            one = run_gpu(w, 2, 1, args.seed, profile=False, act_terms=1) if r["cfg"]["kind"] == "mlp" else None
            others["cfg%d" % w] = dict(workload=workload_name(w, r["cfg"]), steps_per_s=r0["steps_per_s"],
                                       ms_per_sample=r0["ms_per_sample"], path=r0["path"],
                                       kernel_figures_from=r["path"] + " (profiled pass)",
                                       rounds_mean=r0["rounds_mean"],
                                       rounds_max=r0["rounds_max"], roofline_kernel=rf["kernel"],
                                       roofline_frac=rf["frac"], achieved=rf["achieved"], peak=rf["peak"],
                                       unit=rf["unit"], avg_launch_us=rf["avg_launch_us"],
                                       hbm_kernels=hbm_kernels(r),
                                       window_control=dict(steps_per_s=ra["steps_per_s"],
                                                           ms_per_sample=ra["ms_per_sample"],
                                                           rounds_mean=ra["rounds_mean"],
                                                           rounds_max=ra["rounds_max"]))
            if one is not None:
                # the same network with activations rounded to one bf16 term (half the matrix-core work; its
                # outputs agree with any other implementation to ~2e-3 of the unclipped output scale only)
                others["cfg%d" % w]["mlp_activation_terms"] = r["act_terms"]
                others["cfg%d" % w]["one_term_activations"] = dict(steps_per_s=one["steps_per_s"],
                                                                   ms_per_sample=one["ms_per_sample"])
        line["other_workloads"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
