"""GPU parity: the HIP library (through its C boundary) against the CPU oracle,
element by element on the same seeded inputs."""
import numpy as np
import pytest
import torch

import asd_workloads as W
from oracle import asd as oasd
from oracle import philox
from oracle_helpers import chain_randoms, mlp_model, oracle_setup

pytestmark = pytest.mark.gpu

try:
    from paper_2505_03983_amd import binding, probe, runtime
    import gpu_helpers as H
except Exception:  # pragma: no cover - import errors surface in the tests
    raise

DEV = "cuda:0"


def _log(*a):
    print(*a, flush=True)


# ---------------------------------------------------------------------------
# random numbers
# ---------------------------------------------------------------------------
def test_philox_words_bit_identical():
    for seed, chain, step, sid in [(0, 0, 0, 0), (12345, 7, 999, 1), ((1 << 40) + 17, 1023, 1000, 0)]:
        nblk = 300
        out = torch.zeros((nblk, 4), dtype=torch.int32, device=DEV)
        binding.asd_debug_philox(seed, chain, step, sid, nblk, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy().view(np.uint32)
        ctr = np.zeros((nblk, 4), dtype=np.uint64)
        ctr[:, 0] = np.arange(nblk)
        ctr[:, 1], ctr[:, 2], ctr[:, 3] = step, chain, sid
        want = philox.philox4x32_10(ctr, philox.seed_key(seed))
        assert np.array_equal(got, want)


def test_normals_and_uniforms_match_oracle():
    d = 1023
    worst = 0.0
    cases = [(0, 0, 0), (3, 5, 17), (99, 1000, 1000)] + [(7, c, s) for c in range(6) for s in range(1, 40, 3)]
    for seed, chain, step in cases:
        xi = torch.zeros(d, dtype=torch.float32, device=DEV)
        u = torch.zeros(1, dtype=torch.float32, device=DEV)
        binding.asd_debug_randoms(seed, chain, step, d, xi, u)
        torch.cuda.synchronize()
        want = philox.normals(seed, chain, [step], d)[0]
        worst = max(worst, float(np.max(np.abs(xi.cpu().numpy() - want))))
        assert float(u.cpu()[0]) == philox.uniforms(seed, chain, [step])[0]      # exact in fp32
    _log("max |xi_dev - xi_oracle| =", worst)
    assert worst < 5e-6


# ---------------------------------------------------------------------------
# denoisers
# ---------------------------------------------------------------------------
def _denoise_case(cfg, n_rows, seed=0, chains=None, L=None, out_clip=None, split=None):
    T, p, model = oracle_setup(cfg)
    if out_clip is not None:
        p["out_clip"] = out_clip
        model = mlp_model(T, p)
    ctx = runtime.open_ctx(cfg, p, seed=seed, chains=chains, L=L)
    if split is not None:
        ctx.use_split_gemm(split)
        assert ctx.split_gemm_active() == bool(split and cfg["d"] % 16 == 0 and cfg["C"] % 16 == 0)
    rng = np.random.default_rng(seed)
    tau = rng.integers(1, cfg["K"] + 1, n_rows).astype(np.int32)
    ab = T["abar"][tau]
    if cfg["kind"] == "gmm":     # clean samples of the data law: a component mean plus within-component noise
        x0 = p["means"][rng.integers(0, cfg["C"], n_rows)] + np.sqrt(p["var"]) * rng.standard_normal((n_rows, cfg["d"]))
    else:
        x0 = rng.uniform(-1.0, 1.0, (n_rows, cfg["d"]))          # data range of the clipped network
    x = (np.sqrt(ab)[:, None] * x0 + np.sqrt(1 - ab)[:, None] * rng.standard_normal((n_rows, cfg["d"]))).astype(np.float32)
    xd = torch.from_numpy(x).to(DEV)
    out = torch.zeros_like(xd)
    ctx.denoise(xd, torch.from_numpy(tau).to(DEV), out)
    torch.cuda.synchronize()
    want = model(K_minus(tau, cfg["K"]), x.astype(np.float64))
    ctx.close()
    return out.cpu().numpy(), want


def K_minus(tau, K):
    return K - np.asarray(tau)          # step index i with tau[i] = K - i


@pytest.mark.parametrize("shape", [dict(d=2, C=4), dict(d=64, C=256), dict(d=7, C=5), dict(d=3, C=130),
                                   dict(d=4, C=3), dict(d=8, C=5), dict(d=100, C=67), dict(d=256, C=33),
                                   dict(d=260, C=9)])
def test_gmm_rowwise_denoiser(shape):
    cfg = dict(kind="gmm", K=50, chains=4, L=8, var=0.25, **shape)
    got, want = _denoise_case(cfg, 29)
    e = H.rel_err(got, want)
    _log("gmm rowwise", shape, "rel err", e)
    assert e <= 1e-4


@pytest.mark.parametrize("split", [True, False])
@pytest.mark.parametrize("shape", [dict(d=128, C=384, rows=300), dict(d=36, C=132, rows=131), dict(d=1024, C=4096, rows=160),
                                   dict(d=48, C=272, rows=700), dict(d=16, C=16, rows=129)])
def test_gmm_matrix_core_denoiser(shape, split):
    """Both forms of the verify GEMMs (fp32 MFMA; bf16 MFMA on three-way split operands, taken when d and C
    are multiples of 16) against the fp64 oracle, to the same tolerance: ragged last row tile, C and d
    that are not multiples of the tile, one slab of K."""
    shape = dict(shape)
    rows = shape.pop("rows")
    # enough rows*C*d to select the matrix-core path
    chains = max(8, -(-rows // 16), int(np.ceil((1 << 26) / (shape["C"] * shape["d"] * 16))) + 1)
    cfg = dict(kind="gmm", K=50, chains=chains, L=16, var=0.25, **shape)
    got, want = _denoise_case(cfg, rows, split=split)
    e = H.rel_err(got, want)
    _log("gmm mfma", shape, "split", split, "rows", rows, "rel err", e)
    assert e <= 1e-4


@pytest.mark.parametrize("terms", [1, 2])
@pytest.mark.parametrize("shape", [dict(d=8, E=8, width=16, n_blocks=1, rows=5),
                                   dict(d=112, E=128, width=1024, n_blocks=4, rows=200),
                                   dict(d=40, E=24, width=136, n_blocks=2, rows=131),
                                   dict(d=64, E=64, width=2048, n_blocks=1, rows=300, chains=40)])
def test_mlp_denoiser(shape, terms):
    """The network on its own, activations as one bf16 term or as two (the default of the workloads), draft-call
    and verify-call tilings (the last shape's weight matrices are large enough for the K split)."""
    shape = dict(shape)
    rows = shape.pop("rows")
    cfg = dict(dict(kind="mlp", K=20, chains=16, L=16, act_terms=terms), **shape)
    got, want = _denoise_case(cfg, rows)
    e = H.rel_err(got, want)
    _log("mlp", shape, "terms", terms, "rel err", e, "share of clipped outputs", float(np.mean(np.abs(want) >= 1.0)))
    assert e <= 2e-2
    # without the clip (values relative to the output scale): far below the bar; guards against layout
    # slips that a loose bar could hide
    got, want = _denoise_case(cfg, rows, out_clip=0.0)
    e = H.rel_err(got, want)
    _log("mlp unclipped", shape, "terms", terms, "rel err", e, "max |out|", float(np.abs(want).max()))
    assert e <= (5e-3 if terms == 1 else 1e-4)


def test_one_term_activations_at_full_size():
    """act_terms = 1 on the image-shaped network (its own tilings: 128 x 256 tiles): what that mode guarantees
    is the bar relative to the network's output scale -- the 2^-9 rounding of the activations is amplified to
    ~2e-3 of that scale whatever the accumulation order, which on outputs clipped to [-1, 1] is up to 0.05."""
    cfg = dict(W.CONFIGS[4], act_terms=1, chains=16)
    got, want = _denoise_case(cfg, 300, out_clip=0.0)
    e = H.rel_err(got, want)
    _log("cfg 4 network, one-term activations, unclipped: rel err", e, "max |out|", float(np.abs(want).max()))
    assert e <= 5e-3
    _teacher_forced(dict(W.CONFIGS[3], act_terms=1), seed=0, chains_checked=[0, 255], rounds_per_chain=2)


# ---------------------------------------------------------------------------
# one round, teacher-forced from oracle states
# ---------------------------------------------------------------------------
def _teacher_forced(cfg, seed, chains_checked, rounds_per_chain=4, model_seed=1):
    T, p, model = oracle_setup(cfg, model_seed)
    tol = H.TOL[cfg["kind"]]
    ctx = runtime.open_ctx(cfg, p, seed=seed)
    B, K = cfg["chains"], cfg["K"]
    recs = {}
    for c in chains_checked:
        y, R, rounds, xi, u = H.oracle_chain(cfg, T, model, seed, c, eps=tol)
        recs[c] = (y, rounds, xi)
    n_own = n_other = 0
    worst = {}
    for t in range(rounds_per_chain):
        states = []
        picked = {}
        for c in range(B):
            if c in recs:
                y, rounds, _ = recs[c]
                # spread picks over the run: first, middle, late and the final round
                idx = [0, len(rounds) // 2, max(len(rounds) - 2, 0), len(rounds) - 1][t % 4]
                rec = rounds[idx]
                picked[c] = rec
                states.append((rec["a"], y[rec["a"]].astype(np.float32)))
            else:
                states.append((K, np.zeros(cfg["d"], np.float32)))       # finished chain: must stay untouched
        out = H.teacher_forced_round(ctx, cfg, states)
        for c, rec in picked.items():
            own = H.compare_round(out, c, rec, tol, K, T["c_0"], H.unclipped_scale(cfg, T, p, rec), worst, recs[c][2])
            n_own += own
            n_other += (not own)
        for c in range(B):
            if c not in recs:
                assert out["a_next"][c] == K and out["accepted"][c] == -1
                assert not out["traj"][c].any()
    ctx.close()
    _log("teacher-forced", cfg["kind"], "d", cfg["d"], "rounds compared", n_own + n_other,
         "of them on the other branch of a flagged near-tie", n_other, "worst errors",
         {k: float("%.2e" % v) for k, v in worst.items()})
    return worst


def test_noise_predicting_mlp():
    """predict_eps: the network output is turned into x_0 in the last epilogue.  The conversion
    multiplies the output by sqrt(1 - abar)/sqrt(abar) (up to ~10 at K = 20), so unclipped values are
    compared relative to their own scale, clipped ones to the usual bar; then single rounds and whole
    samples against the oracle."""
    cfg = dict(kind="mlp", d=40, E=24, width=136, n_blocks=2, K=20, chains=12, L=6, predict_eps=True)
    got, want = _denoise_case(cfg, 67)
    assert H.rel_err(got, want) <= 2e-2
    got, want = _denoise_case(cfg, 67, out_clip=0.0)
    assert H.rel_err(got, want) <= 5e-3
    _teacher_forced(cfg, seed=11, chains_checked=range(4))
    _free_running(cfg, 11, range(6), resident=False)


def test_round_config1():
    _teacher_forced(W.CONFIGS[1], seed=0, chains_checked=range(8))


def test_round_config2():
    _teacher_forced(W.CONFIGS[2], seed=0, chains_checked=[0, 1, 31, 63])


def test_round_config3_bf16_mlp():
    worst = _teacher_forced(W.CONFIGS[3], seed=0, chains_checked=[0, 100, 255], rounds_per_chain=4)
    assert worst["x0hat"] <= 1e-3          # two-term activations: far inside the 2e-2 bar


def test_round_ragged_shapes():
    # d not a multiple of 4, K not a multiple of L, tiny K
    for cfg in (dict(kind="gmm", d=7, C=5, K=23, chains=5, L=6, var=0.25),
                dict(kind="gmm", d=3, C=9, K=2, chains=3, L=64, var=0.25),
                dict(kind="gmm", d=5, C=3, K=1, chains=2, L=4, var=0.25)):
        _teacher_forced(cfg, seed=5, chains_checked=range(cfg["chains"] - 1))


def test_matrix_core_denoiser_is_deterministic():
    """Repeated calls give bit-identical results on every matrix-core path: split-operand and fp32 verify GEMMs
    (asd_denoise), and the draft call with its K-split second GEMM (partials added in a fixed order)."""
    cfg = dict(kind="gmm", d=48, C=1024, K=30, chains=70, L=24, var=0.25)
    T, p, _ = oracle_setup(cfg)
    ctx = runtime.open_ctx(cfg, p, seed=1)
    rng = np.random.default_rng(4)
    x = torch.from_numpy(rng.standard_normal((900, cfg["d"])).astype(np.float32)).to(DEV)
    tau = torch.from_numpy(rng.integers(1, cfg["K"] + 1, 900).astype(np.int32)).to(DEV)
    for split in (True, False):
        ctx.use_split_gemm(split)
        outs = []
        for _ in range(3):
            out = torch.zeros_like(x)
            ctx.denoise(x, tau, out)
            outs.append(out.clone())
        torch.cuda.synchronize()
        assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2]), split
    # one round from the same states, twice: draft call (K split), draft, verify call, accept
    B, K, L, d = cfg["chains"], cfg["K"], cfg["L"], cfg["d"]
    results = []
    for _ in range(2):
        traj = torch.zeros((B, K + 1, d), dtype=torch.float32, device=DEV)
        traj[:, 0] = torch.arange(B, device=DEV, dtype=torch.float32)[:, None] * 0.01 + 0.3
        a = torch.zeros(B, dtype=torch.int32, device=DEV)
        x0hat = torch.zeros((B, L, d), dtype=torch.float32, device=DEV)
        ctx.draft(traj, a)
        ctx.verify(traj, a, x0hat)
        ctx.accept(traj, a, x0hat)
        torch.cuda.synchronize()
        results.append((traj.clone(), a.clone(), x0hat.clone()))
    for u, v in zip(results[0], results[1]):
        assert torch.equal(u, v)
    ctx.close()


def test_sparse_combine_is_bit_identical_to_the_dense_loop():
    """The second split GEMM skips the slabs of components whose softmax weights are exactly 0.0f for a whole
    row tile.  Rows at all noise levels (broad posteriors early, collapsed ones late), ragged row tile: the
    result must equal the dense loop's bit for bit, and both the oracle's."""
    for cfg, n_rows in ((dict(kind="gmm", d=64, C=1024, K=200, chains=70, L=16, var=0.25), 700),
                        (dict(kind="gmm", d=128, C=4096, K=1000, chains=40, L=16, var=0.25), 517)):
        T, p, model = oracle_setup(cfg)
        ctx = runtime.open_ctx(cfg, p, seed=0)
        assert ctx.split_gemm_active()
        rng = np.random.default_rng(7)
        tau = np.sort(rng.integers(1, cfg["K"] + 1, n_rows)).astype(np.int32)      # tiles of similar noise level
        ab = T["abar"][tau]
        x0 = p["means"][rng.integers(0, cfg["C"], n_rows)] + np.sqrt(p["var"]) * rng.standard_normal((n_rows, cfg["d"]))
        x = (np.sqrt(ab)[:, None] * x0 + np.sqrt(1 - ab)[:, None] * rng.standard_normal((n_rows, cfg["d"]))).astype(np.float32)
        xd, td = torch.from_numpy(x).to(DEV), torch.from_numpy(tau).to(DEV)
        outs = []
        for sparse in (True, False, True):
            ctx.use_sparse_combine(sparse)
            out = torch.zeros_like(xd)
            ctx.denoise(xd, td, out)
            torch.cuda.synchronize()
            outs.append(out)
        assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
        want = model(K_minus(tau, cfg["K"]), x.astype(np.float64))
        e = H.rel_err(outs[0].cpu().numpy(), want)
        _log("sparse combine", cfg["C"], "components: bit-identical to dense, rel err vs oracle", e)
        assert e <= 1e-4
        ctx.close()


def test_logit_screen_is_bit_identical_and_skips_work():
    """The screening pass in front of the verify call's first GEMM (a one-product bf16 GEMM with a rigorous error
    bound) lets the exact GEMM leave out the tiles whose softmax weights are all exactly 0.0f.  (a) Rows at all noise
    levels through the model call alone, ragged row tile, every row of a tile near the same component so that
    tiles do die: always screened == never screened, bit for bit, tiles are left out, and the oracle agrees.
    (b) Whole samples (draft verdict -> screened or not, graphs on): the three modes give the same trajectories and
    round counts bit for bit, and so do samples without the one-hot certificate, which does certify row tiles."""
    cfg = dict(kind="gmm", d=128, C=1024, K=200, chains=72, L=16, var=0.25)
    T, p, model = oracle_setup(cfg)
    ctx = runtime.open_ctx(cfg, p, seed=0)
    assert ctx.split_gemm_active() and ctx.logit_screen_active() == 1
    rng = np.random.default_rng(11)
    n_rows = 1000                                                     # 7 full row tiles and one of 104 rows
    tau = np.sort(rng.integers(1, cfg["K"] + 1, n_rows)).astype(np.int32)
    comp = np.repeat(rng.integers(0, cfg["C"], (n_rows + 127) // 128), 128)[:n_rows]   # one component per row tile
    ab = T["abar"][tau]
    x0 = p["means"][comp] + np.sqrt(p["var"]) * rng.standard_normal((n_rows, cfg["d"]))
    # every other row tile sits half way between two components: two weights survive there, so the tile is not one-hot
    comp2 = np.repeat(rng.integers(0, cfg["C"], (n_rows + 127) // 128), 128)[:n_rows]
    odd = (np.arange(n_rows) // 128) % 2 == 1
    x0[odd] = 0.5 * (p["means"][comp[odd]] + p["means"][comp2[odd]]) + np.sqrt(p["var"]) * rng.standard_normal((int(odd.sum()), cfg["d"]))
    x = (np.sqrt(ab)[:, None] * x0 + np.sqrt(1 - ab)[:, None] * rng.standard_normal((n_rows, cfg["d"]))).astype(np.float32)
    xd, td = torch.from_numpy(x).to(DEV), torch.from_numpy(tau).to(DEV)
    outs, work = [], []
    ctx.profile_enable(True)
    for mode in (2, 0, 2):
        ctx.use_logit_screen(mode)
        assert ctx.logit_screen_active() == mode
        out = torch.zeros_like(xd)
        ctx.denoise(xd, td, out)
        torch.cuda.synchronize()
        outs.append(out)
        work.append(ctx.profile_model_work())
        ctx.profile_enable(True)                                      # clears the counters
    ctx.profile_enable(False)
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    done, tiles = work[0][0], work[0][1]
    assert tiles == 16 * (cfg["C"] // 128) and 16 <= done < tiles and work[0][4] == tiles and work[1][:2] == (0, 0)   # half tiles
    # the second GEMM leaves the same work out either way: whole row tiles to the closed form, slabs of the others
    assert 0 < work[0][2] <= work[0][3] and work[1][2:4] == work[0][2:4] and 0 < work[0][5] < 8 and work[1][5] == work[0][5]
    want = model(K_minus(tau, cfg["K"]), x.astype(np.float64))
    e = H.rel_err(outs[0].cpu().numpy(), want)
    _log("logit screen: %d of %d half tiles computed, bit-identical to unscreened, rel err vs oracle" % (done, tiles), e)
    assert e <= 1e-4
    with pytest.raises(binding.AsdError):
        ctx.use_logit_screen(3)
    ctx.use_logit_screen(1)
    ctx.use_sparse_combine(False)                                     # nothing would skip what the screen leaves out
    assert ctx.logit_screen_active() == 0
    out = torch.zeros_like(xd)
    ctx.denoise(xd, td, out)
    torch.cuda.synchronize()
    assert torch.equal(out, outs[0])
    ctx.use_sparse_combine(True)
    # (b) whole samples: this shape, and the shape of the largest workload with fewer chains (windows of 64: the
    # verify plan then lays the chains' rows out in blocks of 64, repeats of a chain's last row filling its block)
    for cfg_b, ctx_b in ((cfg, ctx), (dict(W.CONFIGS[5], chains=48), None)):
        if ctx_b is None:
            ctx_b = runtime.open_ctx(cfg_b, W.make_params(cfg_b, 1), seed=0)
            assert ctx_b.logit_screen_active() == 1
        res = []
        for mode in (0, 1, 2):
            ctx_b.use_logit_screen(mode)
            ctx_b.set_seed(5)
            traj = runtime.alloc_traj(ctx_b)
            rounds = torch.zeros(cfg_b["chains"], dtype=torch.int32, device=DEV)
            ctx_b.sample(traj, rounds)
            torch.cuda.synchronize()
            res.append((traj, rounds))
        # and with the second GEMM visiting everything (no slab skipped, no row in closed form, hence no screen either)
        ctx_b.use_logit_screen(1)
        ctx_b.use_sparse_combine(False)
        ctx_b.set_seed(5)
        traj = runtime.alloc_traj(ctx_b)
        rounds = torch.zeros(cfg_b["chains"], dtype=torch.int32, device=DEV)
        ctx_b.sample(traj, rounds)
        torch.cuda.synchronize()
        res.append((traj, rounds))
        ctx_b.use_sparse_combine(True)
        # without the one-hot certificate (row tiles proven one-hot before any matrix work), and with it under the
        # profiler (plain launches instead of graphs), which also says how many row tiles it took
        assert ctx_b.onehot_certificate_active()
        ctx_b.use_onehot_certificate(False)
        assert not ctx_b.onehot_certificate_active()
        ctx_b.set_seed(5)
        traj = runtime.alloc_traj(ctx_b)
        rounds = torch.zeros(cfg_b["chains"], dtype=torch.int32, device=DEV)
        ctx_b.sample(traj, rounds)
        torch.cuda.synchronize()
        res.append((traj, rounds))
        ctx_b.use_onehot_certificate(True)
        ctx_b.profile_enable(True)
        ctx_b.set_seed(5)
        traj = runtime.alloc_traj(ctx_b)
        rounds = torch.zeros(cfg_b["chains"], dtype=torch.int32, device=DEV)
        ctx_b.sample(traj, rounds)
        torch.cuda.synchronize()
        res.append((traj, rounds))
        work_b = ctx_b.profile_model_work()
        ctx_b.profile_enable(False)
        assert 0 < work_b[6] <= work_b[5]
        for traj, rounds in res[1:]:
            assert torch.equal(traj, res[0][0]) and torch.equal(rounds, res[0][1])
        assert bool(torch.isfinite(res[0][0]).all())
        _log("logit screen: whole samples of d", cfg_b["d"], "C", cfg_b["C"], "bit-identical in the three modes, with the dense second GEMM and without the certificate; rounds max",
             int(res[0][1].max()), "row tiles in closed form", work_b[5], "of them certified", work_b[6])
        ctx_b.close()


def test_tall_tiles_are_bit_identical_to_the_small_ones():
    """Verify calls of many rows whose every tile is wanted run their GEMMs on 256 x 256 tiles (the same terms in the
    same order per element).  The largest workload's shape with a quarter of its chains -- 16384 model rows per
    call, the least that takes them: whole samples with the tall tiles, without, and without the screening pass
    either way (then every verify call is a dense one, the late ones with rows of one weight among them)."""
    cfg = dict(W.CONFIGS[5], chains=256)
    ctx = runtime.open_ctx(cfg, W.make_params(cfg, 1), seed=0)
    assert ctx.tall_tiles_active() and ctx.logit_screen_active() == 1
    res = []
    for tall, screen in ((True, 1), (False, 1), (True, 0), (False, 0)):
        ctx.use_tall_tiles(tall)
        ctx.use_logit_screen(screen)
        assert ctx.tall_tiles_active() == tall
        ctx.set_seed(9)
        traj = runtime.alloc_traj(ctx)
        rounds = torch.zeros(cfg["chains"], dtype=torch.int32, device=DEV)
        ctx.sample(traj, rounds)
        torch.cuda.synchronize()
        res.append((traj, rounds))
    for traj, rounds in res[1:]:
        assert torch.equal(traj, res[0][0]) and torch.equal(rounds, res[0][1])
    assert bool(torch.isfinite(res[0][0]).all())
    _log("tall tiles: whole samples of 256 chains bit-identical with and without them, screened and not; rounds max", int(res[0][1].max()))
    ctx.close()


def test_mfma_ceiling_probe():
    """The probe of what the matrix pipes sustain: plausible, finite figures (no fixed expectation: the rate is set
    by the chip's power management), constant operands no slower than random ones."""
    r_bf16 = probe.asd_probe_mfma_ceiling(1, True, 60)
    c_bf16 = probe.asd_probe_mfma_ceiling(1, False, 60)
    r_f16 = probe.asd_probe_mfma_ceiling(2, True, 60)
    r_f32 = probe.asd_probe_mfma_ceiling(0, True, 60)
    _log("mfma ceiling: bf16 random", r_bf16, "constant", c_bf16, "fp16 random", r_f16, "f32 random", r_f32)
    assert 200.0 < r_bf16 <= 2600.0 and 200.0 < c_bf16 <= 2600.0 and c_bf16 >= 0.95 * r_bf16
    assert 200.0 < r_f16 <= 2600.0
    assert 40.0 < r_f32 <= 165.0


def test_round_midsize_matrix_core_shapes():
    """Rounds whose two model calls both take the matrix-core path on shapes that are not tile multiples:
    a draft call of 70 rows with its second GEMM split over K (C = 1024, fp32 MFMA: d is not a multiple of 16),
    a shape that takes the split-operand kernels for the verify call only (d = 48, C = 1040: ragged last column
    tile, fp32 draft call without a K split), and two that take them for both calls."""
    for cfg in (dict(kind="gmm", d=40, C=1024, K=30, chains=70, L=24, var=0.25),
                dict(kind="gmm", d=48, C=1040, K=20, chains=90, L=16, var=0.25),
                # both calls on the split-operand kernels: an odd number of 32-wide K slabs and a ragged column tile
                # (no K split), then a ragged row tile with the second GEMM's K split two ways
                dict(kind="gmm", d=96, C=1056, K=20, chains=90, L=8, var=0.25),
                dict(kind="gmm", d=64, C=1024, K=20, chains=70, L=16, var=0.25)):
        _teacher_forced(cfg, seed=2, chains_checked=[0, 33, cfg["chains"] - 1], rounds_per_chain=2)


# ---------------------------------------------------------------------------
# whole samples, free-running
# ---------------------------------------------------------------------------
def _free_running(cfg, seed, chains_checked, y0=None, resident=True, adaptive=False, graphs=True, reuse=False):
    """Whole samples from asd_sample against the oracle's Alg. 1 run next to them (H.follow_chain): every
    chain is compared over all K steps; on a flagged near-tie the oracle follows the branch the device took.
    resident: let asd_sample use the chain-resident kernel where the shape allows (the default);
    False forces the lock-step round kernels.  adaptive: windows from the controller, on both sides.
    Returns the number of chains that needed no such following (the oracle's own run, value for value)."""
    T, p, model = oracle_setup(cfg)
    tol = H.TOL[cfg["kind"]]
    ctx = runtime.open_ctx(cfg, p, seed=seed)
    ctx.use_resident(resident)
    ctx.use_adaptive_window(adaptive)
    ctx.use_graphs(graphs)
    ctx.use_call_reuse(reuse)
    traj = runtime.alloc_traj(ctx)
    rounds = torch.zeros(cfg["chains"], dtype=torch.int32, device=DEV)
    n_launch = ctx.sample(traj, rounds)
    tj, rd = traj.cpu().numpy(), rounds.cpu().numpy()
    if ctx.early_accept_active():
        # a round launched without the kernels behind the early accept kernel may leave a chain waiting for the next
        # full one: a few launches more than the longest chain's rounds
        assert rd.max() <= n_launch <= rd.max() + 8
        ctx.profile_enable(True)                       # (plain launches) the same sample once more, with the counters
        again = runtime.alloc_traj(ctx)
        ctx.sample(again)
        taken = ctx.profile_early_accept()[1]
        ctx.profile_enable(False)
        assert torch.equal(again, traj) and taken > 0
        _log("early accept took", taken, "of", int(rd.sum()), "chain-rounds")
        del again
    else:
        assert n_launch == rd.max()
    full = flips = flagged = 0
    worst = 0.0
    for c in chains_checked:
        f = H.follow_chain(cfg, T, model, seed, c, tj[c], tol, adaptive=adaptive, reuse=reuse)
        e = H.rel_err(tj[c], f["y"])
        worst = max(worst, e)
        assert e <= tol, ("trajectory", c, e)
        assert rd[c] == f["R"], ("rounds", c, rd[c], f["R"])
        full += f["flips"] == 0
        flips += f["flips"]
        flagged += f["flagged_slots"]
    ctx.close()
    _log("free-running", cfg["kind"], "d", cfg["d"], "chains compared over all steps", len(list(chains_checked)),
         "on the oracle's own branches throughout", full, "flagged slots", flagged, "followed to the other branch", flips,
         "worst rel err %.2e" % worst, "rounds mean/max", rd.mean(), rd.max())
    return full


@pytest.mark.parametrize("resident", [False, True])
def test_sample_config1_all_chains(resident):
    full = 0
    for seed in range(4):
        full += _free_running(W.CONFIGS[1], seed, range(8), resident=resident)
    assert full >= 24


@pytest.mark.parametrize("resident", [False, True])
def test_sample_config2_subset(resident):
    assert _free_running(W.CONFIGS[2], 0, [0, 17, 63], resident=resident) >= 1


@pytest.mark.parametrize("resident", [False, True])
def test_sample_ragged_shapes(resident):
    """Whole samples on shapes with d not a multiple of 4, C not a multiple of 4 or 64, windows cut
    by K, L = 64 and a single chain."""
    for cfg in (dict(kind="gmm", d=7, C=5, K=37, chains=5, L=6, var=0.25),
                dict(kind="gmm", d=3, C=130, K=70, chains=3, L=64, var=0.25),
                dict(kind="gmm", d=20, C=66, K=25, chains=1, L=9, var=0.25),
                dict(kind="gmm", d=5, C=3, K=1, chains=2, L=4, var=0.25)):
        full = _free_running(cfg, 6, range(cfg["chains"]), resident=resident)
        assert full >= 1


def test_windows_longer_than_64_and_asd_infinity():
    """L > 64 (the first-rejection scan walks the window in groups) and L >= K (the paper's
    ASD-infinity: every round speculates to the end of the chain), as single rounds and whole samples."""
    big = dict(kind="gmm", d=8, C=6, K=150, chains=4, L=100, var=0.25)
    _teacher_forced(big, seed=8, chains_checked=range(3))
    assert _free_running(big, 8, range(4)) >= 1
    inf = dict(W.CONFIGS[1], L=W.CONFIGS[1]["K"])
    _teacher_forced(inf, seed=9, chains_checked=range(4))
    assert _free_running(inf, 9, range(8)) >= 4
    wide = dict(kind="gmm", d=132, C=40, K=90, chains=3, L=130, var=0.25)      # matrix-core or row-wise GMM path
    assert _free_running(wide, 10, range(3)) >= 1


@pytest.mark.parametrize("resident", [False, True])
def test_adaptive_windows_match_the_oracle(resident):
    """Windows chosen by the controller from each chain's past: same integer rule on both sides, so
    rounds, windows and trajectories must agree with the oracle as for fixed windows."""
    full = 0
    for seed in range(2):
        full += _free_running(W.CONFIGS[1], 30 + seed, range(8), resident=resident, adaptive=True)
    assert full >= 12
    assert _free_running(W.CONFIGS[2], 32, [0, 5, 63], resident=resident, adaptive=True) >= 1
    ragged = dict(kind="gmm", d=7, C=5, K=61, chains=5, L=40, var=0.25)
    assert _free_running(ragged, 33, range(5), resident=resident, adaptive=True) >= 1
    if not resident:
        small_mlp = dict(kind="mlp", d=16, E=8, width=64, n_blocks=2, K=30, chains=6, L=12)
        _free_running(small_mlp, 34, range(6), resident=False, adaptive=True)
        # weight matrices large enough (8 MB) that verify calls far below their row bound are routed,
        # on the device, to the small-row tile shape: windows of 4 give 120 rows, windows of 9 give 320
        wide_mlp = dict(kind="mlp", d=64, E=64, width=2048, n_blocks=1, K=14, chains=40, L=12)
        _free_running(wide_mlp, 35, [0, 7, 39], resident=False, adaptive=True)
        _free_running(wide_mlp, 35, [1, 38], resident=False, adaptive=False)


def test_adaptive_windows_save_model_rows_and_toggle_cleanly():
    """On a workload whose windows are mostly rejected early the controller must cut the verify rows;
    switching it off again restores the fixed-window sample bit for bit (the round graph is rebuilt)."""
    cfg = W.CONFIGS[2]
    _, p, _ = oracle_setup(cfg)
    ctx = runtime.open_ctx(cfg, p, seed=5)
    ctx.use_resident(False)
    t0, t1, t2 = (runtime.alloc_traj(ctx) for _ in range(3))
    r0 = torch.zeros(cfg["chains"], dtype=torch.int32, device=DEV)
    r1, r2 = torch.zeros_like(r0), torch.zeros_like(r0)
    ctx.sample(t0, r0)
    ctx.use_adaptive_window(True)
    ctx.sample(t1, r1)
    ctx.use_adaptive_window(False)
    ctx.sample(t2, r2)
    assert torch.equal(t0, t2) and torch.equal(r0, r2)
    assert torch.isfinite(t1).all()
    ctx.profile_enable(True)
    ctx.sample(t2, r2)
    fixed_rows = ctx.profile_rows()[1]
    ctx.profile_enable(False)
    ctx.use_adaptive_window(True)
    ctx.profile_enable(True)
    ctx.sample(t1, r1)
    adaptive_rows = ctx.profile_rows()[1]
    ctx.profile_enable(False)
    _log("verify rows per sample: fixed", fixed_rows, "adaptive", adaptive_rows, "rounds max", int(r2.max()), int(r1.max()))
    assert adaptive_rows < fixed_rows
    ctx.close()


def test_early_accept_is_bit_identical_and_takes_chains():
    """asd_use_early_accept: chains whose rows the one-hot certificate covers have their accept stage ahead of the
    verify call, on model values the accept kernel forms itself.  Whole samples of the largest workload's shape (fewer
    chains, but enough rows that the row plans are made by the planning kernels) with it on and off: the same
    trajectories and round counts bit for bit, fixed windows and controlled ones, rounds as graphs and as plain
    launches; it does take chain-rounds; the drafted rows counted are the same either way."""
    cfg = dict(W.CONFIGS[5], chains=320)
    ctx = runtime.open_ctx(cfg, W.make_params(cfg, 1), seed=0)
    assert ctx.early_accept_active() and ctx.onehot_certificate_active()
    traj = [runtime.alloc_traj(ctx) for _ in range(2)]
    rounds = [torch.zeros(cfg["chains"], dtype=torch.int32, device=DEV) for _ in range(2)]
    for adaptive in (False, True):
        ctx.use_adaptive_window(adaptive)
        for plain in (False, True):
            rows = []
            for i, early in enumerate((True, False)):
                ctx.use_early_accept(early)
                assert ctx.early_accept_active() == early
                ctx.set_seed(7)
                if plain:
                    ctx.profile_enable(True)
                ctx.sample(traj[i], rounds[i])
                torch.cuda.synchronize()
                if plain:
                    rows.append((ctx.profile_rows(), ctx.profile_accept_rows(), ctx.profile_early_accept()))
                    ctx.profile_enable(False)
            assert torch.equal(traj[0], traj[1]) and torch.equal(rounds[0], rounds[1]), (adaptive, plain)
            assert torch.isfinite(traj[0][:, -1]).all()
            if plain:
                (rows_on, acc_on, early_on), (rows_off, acc_off, early_off) = rows
                _log("early accept, adaptive", adaptive, ": model rows formed in the accept kernel", early_on[0],
                     "chain-rounds", early_on[1], "of", int(rounds[0].sum()), "; verify rows", rows_on[1])
                assert early_off == (0, 0, 0, 0) and early_on[1] > int(rounds[0].sum()) // 4 and 0 < early_on[0] <= early_on[2]
                assert 0 < early_on[3] <= early_on[1] and early_on[3] <= acc_on[1]
                # the windows verified are the same; the draft call may see a few chain-rounds more: a chain the
                # early kernel could not take in a round launched without the kernels behind it waits for the next full one
                assert rows_on[1] == rows_off[1] and acc_on == acc_off
                assert rows_off[0] <= rows_on[0] <= rows_off[0] + rows_off[0] // 100
    ctx.use_early_accept(True)
    ctx.use_adaptive_window(False)
    # ... and it stays out of the way where it does not apply
    ctx.use_call_reuse(True)
    assert not ctx.early_accept_active()
    ctx.use_call_reuse(False)
    ctx.use_onehot_certificate(False)
    assert not ctx.early_accept_active()
    ctx.close()
    small = runtime.open_ctx(dict(W.CONFIGS[5], chains=48), W.make_params(dict(W.CONFIGS[5], chains=48), 1), seed=0)
    assert not small.early_accept_active()      # plans folded into the round kernels
    small.close()


def test_early_accept_sample_matches_the_oracle():
    """Whole samples with the early accept kernel at work (a mixture whose late rows certify, enough rows that the
    planning kernels make the plans) against the oracle's Alg. 1, chain by chain over all K steps: fixed windows and
    controlled ones, rounds as graphs and as plain launches."""
    cfg = dict(kind="gmm", d=128, C=256, K=200, chains=272, L=64, var=0.25)
    full = _free_running(cfg, 31, [0, 135, 271], resident=False)
    full += _free_running(cfg, 32, [7, 200], resident=False, adaptive=True)
    full += _free_running(cfg, 33, [64], resident=False, graphs=False)
    assert full >= 4
    # windows longer than a wavefront has lanes (the walk goes on chunk by chunk), one wavefront per chain; and
    # windows that are no multiple of 64 (no chain blocks in the verify plan)
    long_w = dict(kind="gmm", d=256, C=256, K=300, chains=70, L=256, var=0.25)
    assert _free_running(long_w, 41, [0, 69], resident=False) >= 1
    short_w = dict(kind="gmm", d=128, C=512, K=90, chains=600, L=32, var=0.25)
    assert _free_running(short_w, 43, [0, 599], resident=False) >= 1


def test_profile_select_times_the_chosen_slots_only():
    """asd_profile_select: only the selected scopes take events, the work counters run regardless, and the sample
    is the same with any selection."""
    cfg = W.CONFIGS[2]
    _, p, _ = oracle_setup(cfg)
    ctx = runtime.open_ctx(cfg, p, seed=5)
    ctx.use_resident(False)
    t0, t1 = runtime.alloc_traj(ctx), runtime.alloc_traj(ctx)
    P = binding.PROF
    ctx.profile_enable(True)
    ctx.sample(t0)
    every = {(k, c): ctx.profile_read(P[k], c)[0] for k in ("DRAFT", "ACCEPT", "GMM_ROWWISE") for c in (0, 1)}
    rows_all = ctx.profile_rows()
    ctx.profile_select(["GMM_ROWWISE/verify"])
    ctx.profile_enable(True)
    ctx.sample(t1)
    some = {(k, c): ctx.profile_read(P[k], c)[0] for k in ("DRAFT", "ACCEPT", "GMM_ROWWISE") for c in (0, 1)}
    rows_some = ctx.profile_rows()
    ctx.profile_enable(False)
    ctx.profile_select(None)
    assert every[("DRAFT", 0)] > 0 and every[("ACCEPT", 0)] > 0 and every[("GMM_ROWWISE", 0)] > 0
    assert some[("GMM_ROWWISE", 1)] == every[("GMM_ROWWISE", 1)] > 0
    assert all(n == 0 for key, n in some.items() if key != ("GMM_ROWWISE", 1))
    assert rows_some == rows_all and rows_all[1] > 0
    assert torch.equal(t0, t1)
    ctx.close()


def test_model_call_reuse_matches_the_oracle():
    """asd_use_call_reuse: the verify call also evaluates yhat_b, a fully accepted window hands that value to the
    next round and the chain skips the next draft call.  Whole samples against the oracle run with the same rule,
    on the lock-step round kernels: row-wise and matrix-core mixture paths, L = 1 (every round hands over),
    L >= K, windows from the controller, the MLP; rounds as graphs and as plain launches."""
    full = 0
    for seed in range(2):
        full += _free_running(W.CONFIGS[1], 60 + seed, range(8), resident=False, reuse=True)
    assert full >= 12
    _free_running(W.CONFIGS[2], 62, [0, 9, 63], resident=False, reuse=True, adaptive=True)
    for cfg in (dict(kind="gmm", d=7, C=5, K=37, chains=5, L=6, var=0.25),
                dict(kind="gmm", d=5, C=3, K=9, chains=3, L=1, var=0.25),
                dict(W.CONFIGS[1], L=W.CONFIGS[1]["K"]),
                dict(kind="gmm", d=8, C=6, K=150, chains=4, L=100, var=0.25),
                dict(kind="gmm", d=64, C=1024, K=20, chains=70, L=16, var=0.25)):      # matrix-core path, both calls
        _free_running(cfg, 63, range(min(cfg["chains"], 4)), resident=False, reuse=True, graphs=bool(cfg["d"] & 1))
    small_mlp = dict(kind="mlp", d=16, E=8, width=64, n_blocks=2, K=30, chains=6, L=12)
    _free_running(small_mlp, 64, range(6), resident=False, reuse=True)
    _free_running(small_mlp, 64, range(6), resident=False, reuse=True, adaptive=True)
    # the switch changes which call evaluates a row, not the sample: same seed with and without
    cfg = W.CONFIGS[2]
    _, p, _ = oracle_setup(cfg)
    ctx = runtime.open_ctx(cfg, p, seed=5)
    ctx.use_resident(False)
    t0, t1 = runtime.alloc_traj(ctx), runtime.alloc_traj(ctx)
    r0 = torch.zeros(cfg["chains"], dtype=torch.int32, device=DEV)
    r1 = torch.zeros_like(r0)
    ctx.profile_enable(True)
    ctx.sample(t0, r0)
    rows0 = ctx.profile_rows()
    ctx.profile_enable(False)
    ctx.use_call_reuse(True)
    ctx.profile_enable(True)
    ctx.sample(t1, r1)
    rows1 = ctx.profile_rows()
    ctx.profile_enable(False)
    _log("model rows per sample (draft call, verify call): without reuse", rows0, "with", rows1)
    assert torch.equal(r0, r1) and H.rel_err(t1.cpu().numpy(), t0.cpu().numpy()) <= 1e-4
    assert rows1[0] < rows0[0] and rows1[1] > rows0[1]
    ctx.use_call_reuse(False)
    ctx.sample(t1, r1)
    assert torch.equal(t0, t1)
    ctx.close()


@pytest.mark.parametrize("grid", ["ddpm", "ve"])
@pytest.mark.parametrize("resident", [False, True])
def test_sample_in_sl_coordinates(resident, grid):
    """The paper's own coordinates: the Euler chain of Eq. euler-sde on the stochastic-localization
    process (c_x = 1, c_0 = eta_i, sigma = sqrt(eta_i)) with the mean function m(t, y) of Eq. sl-defn as
    the model, given to the library as tables (asd_schedule_sl_euler) plus the SL time of every index.
    Whole samples against the oracle run in the same coordinates; y_0 ~ N(0, t_0 I) is passed in
    (the law of the process at t_0 up to the t_0 x* term, which is negligible at a small t_0).
    grid "ddpm": the times of the linear-beta DDPM chain, t = abar / (1 - abar); "ve": a
    variance-exploding diffusion x = x_0 + s eps, s geometric from 30 down to 0.05, i.e. t = 1 / s^2."""
    from oracle import denoisers, schedule
    K, d, C, L, chains, seed = 60, 6, 5, 8, 6, 12
    p = W.gmm_params(d, C)
    if grid == "ddpm":
        t_grid = schedule.sl_tables(K)["t"]                      # K times -> K - 1 steps
    else:
        t_grid = 1.0 / np.geomspace(30.0, 0.05, K) ** 2
    Km = K - 1
    sched = binding.asd_schedule_sl_euler(t_grid)
    eta64 = np.diff(t_grid)
    np.testing.assert_allclose(sched["c_0"], eta64, rtol=2e-7)
    np.testing.assert_allclose(sched["sigma"], np.sqrt(eta64), rtol=2e-7)
    assert np.all(sched["c_x"] == 1.0) and np.array_equal(sched["tau"], np.arange(Km))
    den = runtime.device_params(dict(kind="gmm", d=d, C=C), p)
    den["n_tau"] = K
    den["sl_time"] = sched["sl_time"]
    ctx = binding.Ctx(sched, den, L, chains, seed)
    ctx.use_resident(resident)
    S = dict(gamma=[np.sqrt(t_grid[0])])
    A64, B64, S64 = sched["c_x"].astype(np.float64), sched["c_0"].astype(np.float64), sched["sigma"].astype(np.float64)
    t64 = den["sl_time"].astype(np.float64)

    def model_sl(idx, rows):
        return denoisers.gmm_sl_mean(rows, t64[np.asarray(idx)], p["means"], p["log_w"], p["var"])

    y0 = np.empty((chains, d), np.float32)
    for c in range(chains):
        xi, _ = chain_randoms(seed, c, Km, d)
        y0[c] = (S["gamma"][0] * xi[0]).astype(np.float32)
    traj = runtime.alloc_traj(ctx)
    rounds = torch.zeros(chains, dtype=torch.int32, device=DEV)
    ctx.sample(traj, rounds, y0=torch.from_numpy(y0).to(DEV))
    tj, rd = traj.cpu().numpy(), rounds.cpu().numpy()
    full = 0
    sl_cfg, sl_T = dict(K=Km, d=d, L=L), dict(c_x=A64, c_0=B64, sigma=S64)
    for c in range(chains):
        f = H.follow_chain(sl_cfg, sl_T, model_sl, seed, c, tj[c], 1e-4, y0=y0[c].astype(np.float64))
        # SL states grow like t (up to ~1e4 here): the bar is relative to the largest state compared
        assert H.rel_err(tj[c], f["y"]) <= 1e-4, c
        assert rd[c] == f["R"]
        full += f["flips"] == 0
    assert full >= 3
    ctx.close()


@pytest.mark.parametrize("resident", [False, True])
def test_many_chains_small_problem(resident):
    """A batch far wider than the machine (20000 chains: several workgroups per CU for the chain-resident
    kernel, twenty scan chunks for the row planner), windows cut by K; sampled chains against the oracle."""
    cfg = dict(kind="gmm", d=4, C=3, K=9, chains=20000, L=4, var=0.25)
    assert _free_running(cfg, 50, [0, 1, 1023, 1024, 9999, 19999], resident=resident) >= 3


@pytest.mark.parametrize("resident", [False, True])
def test_sample_with_a_cosine_schedule(resident):
    """Another variance-preserving schedule through the same tables (asd_abar_cosine + asd_schedule_from_abar):
    its last steps have betas up to 0.999, i.e. a very different noise profile from the linear one."""
    cfg = dict(kind="gmm", d=12, C=9, K=80, chains=6, L=10, var=0.25, schedule="cosine")
    assert _free_running(cfg, 3, range(6), resident=resident) >= 4


def test_sample_random_small_shapes():
    """A seeded sweep over small mixture shapes (d, C, K, L, chains drawn at random, windows fixed or
    controlled, either sampling path): whole samples against the oracle."""
    rng = np.random.default_rng(2024)
    total = 0
    for case in range(10):
        cfg = dict(kind="gmm", var=0.25, d=int(rng.integers(1, 40)), C=int(rng.integers(1, 90)),
                   K=int(rng.integers(1, 60)), L=int(rng.integers(1, 70)), chains=int(rng.integers(1, 6)))
        resident, adaptive = bool(case & 1), bool(case & 2)
        total += _free_running(cfg, 40 + case, range(cfg["chains"]), resident=resident, adaptive=adaptive)
    assert total >= 10


def test_resident_sampler_agrees_with_round_kernels():
    """One launch per sample against the lock-step rounds: same counters and formulas, so chains
    agree to rounding unless a near-tie decision falls differently (rare; those chains differ in
    their round counts and are only counted)."""
    for w, seed in ((1, 21), (2, 22)):
        cfg = W.CONFIGS[w]
        _, p, _ = oracle_setup(cfg)
        ctx = runtime.open_ctx(cfg, p, seed=seed)
        tr, tk = runtime.alloc_traj(ctx), runtime.alloc_traj(ctx)
        rr = torch.zeros(cfg["chains"], dtype=torch.int32, device=DEV)
        rk = torch.zeros_like(rr)
        ctx.use_resident(True)
        n_r = ctx.sample(tr, rr)
        ctx.use_resident(False)
        ctx.sample(tk, rk)
        assert n_r == int(rr.max())
        same = (rr == rk).cpu().numpy()
        assert same.mean() >= 0.9, (w, same.mean())
        a, b = tr.cpu().numpy()[same], tk.cpu().numpy()[same]
        assert H.rel_err(a, b) <= 1e-4, (w, H.rel_err(a, b))
        # a second resident sample of the same seed is bit-identical
        t2 = runtime.alloc_traj(ctx)
        ctx.use_resident(True)
        ctx.sample(t2)
        assert torch.equal(t2, tr)
        ctx.close()


def test_sample_is_deterministic_and_chain_local():
    cfg = W.CONFIGS[2]
    T, p, _ = oracle_setup(cfg)
    ctx = runtime.open_ctx(cfg, p, seed=3)
    t1, t2 = runtime.alloc_traj(ctx), runtime.alloc_traj(ctx)
    r1 = torch.zeros(cfg["chains"], dtype=torch.int32, device=DEV)
    r2 = torch.zeros_like(r1)
    ctx.sample(t1, r1)
    ctx.sample(t2, r2)
    assert torch.equal(t1, t2) and torch.equal(r1, r2)
    ctx.close()
    # a batch of 5 chains reproduces the first 5 chains of the batch of 64 (counter keyed by chain id)
    ctx5 = runtime.open_ctx(cfg, p, seed=3, chains=5)
    t5 = runtime.alloc_traj(ctx5)
    ctx5.sample(t5)
    assert torch.equal(t5, t1[:5])
    ctx5.close()


def test_graph_rounds_equal_plain_launches():
    """The captured per-round graph is replayed many times, with eager work (other samples, other
    contexts, synchronisations) in between; every replayed sample must equal the plainly launched one."""
    for w in (1, 2, 3):
        cfg = W.CONFIGS[w]
        _, p, _ = oracle_setup(cfg)
        ctx = runtime.open_ctx(cfg, p, seed=0)
        ctx.use_resident(False)                        # the rounds are what is under test here
        tg, te = runtime.alloc_traj(ctx), runtime.alloc_traj(ctx)
        rg = torch.zeros(cfg["chains"], dtype=torch.int32, device=DEV)
        re_ = torch.zeros_like(rg)
        side = torch.cuda.Stream()
        for i, seed in enumerate((11, 12, 11, 13)):
            ctx.set_seed(seed)
            ctx.use_graphs(True)
            if i % 2:
                with torch.cuda.stream(side):          # a capturable stream
                    ng = ctx.sample(tg, rg)
                side.synchronize()
            else:
                ng = ctx.sample(tg, rg)                # torch's default stream (the library uses its own)
            ctx.use_graphs(False)
            ne = ctx.sample(te, re_)
            torch.cuda.synchronize()
            assert ng == ne
            assert torch.equal(tg, te) and torch.equal(rg, re_), (w, seed)
        ctx.close()


def test_L1_equals_sequential_sampler_bitwise():
    cfg = dict(W.CONFIGS[1], L=1)
    T, p, model = oracle_setup(cfg)
    ctx = runtime.open_ctx(cfg, p, seed=2)
    ta, ts = runtime.alloc_traj(ctx), runtime.alloc_traj(ctx)
    rounds = torch.zeros(cfg["chains"], dtype=torch.int32, device=DEV)
    ctx.use_resident(False)
    ctx.sample(ta, rounds)
    ctx.sample_sequential(ts)
    assert torch.equal(ta, ts)
    assert (rounds.cpu().numpy() == cfg["K"]).all()
    # the chain-resident kernel walks the same chain (its reductions round differently)
    ctx.use_resident(True)
    ctx.sample(ta, rounds)
    assert H.rel_err(ta.cpu().numpy(), ts.cpu().numpy()) <= 1e-4
    assert (rounds.cpu().numpy() == cfg["K"]).all()
    for c in (0, 7):
        xi, _ = chain_randoms(2, c, cfg["K"], cfg["d"])
        ys = oasd.sequential_chain(xi[0], T["c_x"], T["c_0"], T["sigma"], model, xi)
        assert H.rel_err(ts[c].cpu().numpy(), ys) <= 1e-4
    ctx.close()


def test_given_y0_and_sigma_zero_last_step():
    cfg = W.CONFIGS[1]
    T, p, model = oracle_setup(cfg)
    ctx = runtime.open_ctx(cfg, p, seed=4)
    y0 = torch.full((cfg["chains"], cfg["d"]), 0.5, dtype=torch.float32, device=DEV)
    traj = runtime.alloc_traj(ctx)
    ctx.sample(traj, y0=y0)
    tj = traj.cpu().numpy()
    assert (tj[:, 0] == 0.5).all()
    # last step is deterministic: y_K = c_x y_{K-1} + c_0 D(y_{K-1})
    K = cfg["K"]
    g = model([K - 1] * cfg["chains"], tj[:, K - 1].astype(np.float64))
    want = T["c_x"][K - 1] * tj[:, K - 1] + T["c_0"][K - 1] * g
    assert H.rel_err(tj[:, K], want) <= 1e-4
    ctx.close()


def test_stage_order_is_enforced():
    cfg = W.CONFIGS[1]
    _, p, _ = oracle_setup(cfg)
    ctx = runtime.open_ctx(cfg, p)
    traj = runtime.alloc_traj(ctx)
    a = torch.zeros(cfg["chains"], dtype=torch.int32, device=DEV)
    x0 = torch.zeros((cfg["chains"], cfg["L"], cfg["d"]), dtype=torch.float32, device=DEV)
    with pytest.raises(binding.AsdError) as ei:
        ctx.verify(traj, a, x0)
    assert ei.value.status == binding.ASD_ESTATE
    traj.zero_()
    ctx.draft(traj, a)
    with pytest.raises(binding.AsdError):
        ctx.draft(traj, a)
    ctx.verify(traj, a, x0)
    ctx.accept(traj, a, x0)
    torch.cuda.synchronize()
    ctx.close()


# ---------------------------------------------------------------------------
# full-size workloads in the launch configuration bench.py times
# ---------------------------------------------------------------------------
_SETUPS = {}


def _workload_setup(w):
    """(tables, parameters, oracle model) of workload w, built once per test process (the image-shaped
    network's weights take ten seconds to draw)."""
    if w not in _SETUPS:
        _SETUPS[w] = oracle_setup(W.CONFIGS[w])
    return _SETUPS[w]


def _round_invariants(a_host, a_next, acc, K, L):
    """Structure of a round on every chain (correctness lemma: slot a+1 accepted; advance rule of Alg. 1)."""
    for c in range(len(a_host)):
        if a_host[c] >= K:
            assert a_next[c] == K and acc[c] == -1
            continue
        wdw = min(L, K - a_host[c])
        assert 1 <= acc[c] <= wdw
        assert a_next[c] == a_host[c] + (acc[c] + 1 if acc[c] < wdw else wdw)


def _full_size_round(w, sampled, seed=0, split=None, states=None):
    """One round of workload w with every chain of the batch live, sampled chains against the oracle in full
    (proposal samples, model values, the accept test's sums and ratio, decisions, written rows), all chains
    against the round invariants.  states: (a [B], y_a [B, d]) to start from; default: synthetic mid-run
    states (start, middle, a window cut by K, a finished chain) drawn from the forward marginals."""
    cfg = W.CONFIGS[w]
    T, p, model = _workload_setup(w)
    tol = H.TOL[cfg["kind"]]
    B, K, L, d = cfg["chains"], cfg["K"], cfg["L"], cfg["d"]
    ctx = runtime.open_ctx(cfg, p, seed=seed)
    if split is not None:
        ctx.use_split_gemm(split)
        assert ctx.split_gemm_active() == split
    if states is None:
        rng = np.random.default_rng(seed + 100 * w)
        choices = np.array([0, K // 3, (2 * K) // 3, K - L // 2, K - 1, K])
        a_host = choices[rng.integers(0, len(choices), B)].astype(np.int32)
        a_host[list(sampled)] = [0, K // 3, K - L // 2, (2 * K) // 3][: len(sampled)]
        ya = np.zeros((B, d), np.float32)
        for c in range(B):
            if a_host[c] >= K:
                continue
            ab = T["abar"][T["tau"][a_host[c]]]
            if cfg["kind"] == "gmm":
                x0 = p["means"][rng.integers(0, cfg["C"])] + np.sqrt(p["var"]) * rng.standard_normal(d)
            else:
                x0 = rng.uniform(-1, 1, d)
            ya[c] = np.sqrt(ab) * x0 + np.sqrt(1 - ab) * rng.standard_normal(d)
    else:
        a_host, ya = np.asarray(states[0], np.int32), np.asarray(states[1], np.float32)
    traj = torch.zeros((B, K + 1, d), dtype=torch.float32, device=DEV)
    idx = torch.arange(B, device=DEV)
    a_dev = torch.from_numpy(a_host).to(DEV)
    traj[idx, a_dev.long().clamp(max=K)] = torch.from_numpy(ya).to(DEV)
    x0hat = torch.zeros((B, L, d), dtype=torch.float32, device=DEV)
    accepted = torch.zeros(B, dtype=torch.int32, device=DEV)
    stats = torch.zeros((B, L, 4), dtype=torch.float32, device=DEV)
    a_run = a_dev.clone()
    ctx.draft(traj, a_run)
    ctx.verify(traj, a_run, x0hat)
    drafted = {c: traj[c].cpu().numpy().copy() for c in sampled}
    ctx.accept(traj, a_run, x0hat, accepted, stats)
    torch.cuda.synchronize()
    a_next, acc = a_run.cpu().numpy(), accepted.cpu().numpy()
    _round_invariants(a_host, a_next, acc, K, L)
    assert torch.isfinite(x0hat[torch.from_numpy(a_host < K).to(DEV), 0]).all()
    own = 0
    worst = {}
    for c in sampled:
        xi, u = chain_randoms(seed, c, K, d)
        _log("oracle round", w, "chain", c, "a", int(a_host[c]))
        rec = oasd.asd_round(ya[c].astype(np.float64), int(a_host[c]), L, T["c_x"], T["c_0"], T["sigma"], model, xi, u,
                             eps=tol)
        out = dict(drafted={c: drafted[c]}, x0hat={c: x0hat[c].cpu().numpy()}, accepted={c: acc[c]},
                   a_next={c: a_next[c]}, traj={c: traj[c].cpu().numpy()}, stats={c: stats[c].cpu().numpy()})
        own += bool(H.compare_round(out, c, rec, tol, K, T["c_0"], H.unclipped_scale(cfg, T, p, rec), worst, xi))
    ctx.close()
    _log("full-size round cfg", w, "chains compared in full", len(sampled), "on the oracle's own branch", own,
         "mean accepted", float(acc[acc >= 0].mean()), "worst errors", {k: float("%.2e" % v) for k, v in worst.items()})


def _full_size_prefix(w, seed, chains_checked, n_rounds, adaptive, reuse=False):
    """The whole-sample driver at full size, in the launch configuration the benchmark times: sampled chains of
    a complete asd_sample against the oracle run freely from y_0 for n_rounds rounds (a whole chain would take the
    CPU minutes at these sizes), following the device through flagged near-ties."""
    cfg = W.CONFIGS[w]
    T, p, model = _workload_setup(w)
    tol = H.TOL[cfg["kind"]]
    ctx = runtime.open_ctx(cfg, p, seed=seed)
    ctx.use_adaptive_window(adaptive)
    ctx.use_call_reuse(reuse)
    assert not ctx.resident_active()
    if cfg["kind"] == "gmm":
        assert ctx.split_gemm_active()
    traj = runtime.alloc_traj(ctx)
    rounds = torch.zeros(cfg["chains"], dtype=torch.int32, device=DEV)
    ctx.sample(traj, rounds)
    assert bool(torch.isfinite(traj[:, -1]).all().item())
    steps = 0
    for c in chains_checked:
        tj = traj[c].cpu().numpy()
        f = H.follow_chain(cfg, T, model, seed, c, tj, tol, adaptive=adaptive, max_rounds=n_rounds, reuse=reuse)
        e = H.rel_err(tj[: f["a"] + 1], f["y"][: f["a"] + 1])
        _log("cfg", w, "free-running prefix: chain", c, "adaptive", adaptive, "rounds", f["R"], "steps compared", f["a"],
             "rel err %.2e" % e, "flagged slots", f["flagged_slots"], "followed to the other branch", f["flips"])
        assert e <= tol, (c, f["a"], e)
        steps += f["a"]
    ctx.close()
    return steps


@pytest.mark.parametrize("adaptive", [False, True])
def test_sample_config5_full_size_prefix(adaptive):
    """Headline size (lock-step round kernels, bf16 split-operand verify GEMMs): two chains of a full
    1024-chain sample, five rounds each from y_0."""
    assert _full_size_prefix(5, 3, (0, 777), 5, adaptive) >= 10


def test_model_call_reuse_at_full_size():
    """The two large workloads with model-call reuse and window control on (where handing over pays most)."""
    assert _full_size_prefix(5, 4, (1, 1000), 5, True, reuse=True) >= 10
    assert _full_size_prefix(4, 5, (2, 50), 6, True, reuse=True) >= 12
    assert _full_size_prefix(4, 5, (3,), 6, False, reuse=True) >= 6


def test_round_config4_full_size_sampled():
    _full_size_round(4, sampled=[0, 31, 63])


@pytest.mark.parametrize("split", [True, False])
def test_round_config5_full_size_sampled(split):
    _full_size_round(5, sampled=[0, 517, 1023], split=split)


# ---------------------------------------------------------------------------
# the two MLP workloads end to end (the while-loop of Alg. 1 through asd_sample: round graphs, row plans
# appended by the draft / accept kernels, device-side routing of small verify calls)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("adaptive", [False, True])
def test_sample_config3_whole_chains(adaptive):
    """Diffusion-policy shape at full size: whole samples (all 100 steps) of six chains of the 256-chain batch,
    rounds as captured graphs, fixed windows and windows from the controller."""
    _free_running(W.CONFIGS[3], 0, [0, 1, 100, 177, 254, 255], resident=False, adaptive=adaptive, graphs=True)


def test_sample_config3_plain_launches():
    _free_running(W.CONFIGS[3], 1, [0, 128, 255], resident=False, graphs=False)


@pytest.mark.parametrize("adaptive", [False, True])
def test_sample_config4_full_size_prefix(adaptive):
    """Image-shaped network at full size: two chains of a complete 64-chain sample, six rounds each from y_0."""
    assert _full_size_prefix(4, 2, (0, 63), 6, adaptive) >= 12


def test_round_config4_from_the_oracles_own_chain():
    """Rounds of the image-shaped workload from states of the oracle's own Alg. 1 run (chain 0 to the end, about a
    minute of CPU): the first round, a middle one and the one whose window ends at K (the late states, where
    c_0 -> 1 and most outputs sit on the clip).  Each of the three rounds runs at full size -- every chain of the
    batch starts from one of the three states -- and three chains per round are compared with the oracle in full."""
    cfg = W.CONFIGS[4]
    T, p, model = _workload_setup(4)
    B, K, L = cfg["chains"], cfg["K"], cfg["L"]
    y, R, recs, _, _ = H.oracle_chain(cfg, T, model, 0, 0, eps=H.TOL["mlp"])
    last = next(i for i, r in enumerate(recs) if r["b"] == K)
    picks = [recs[0]["a"], recs[len(recs) // 2]["a"], recs[last]["a"]]
    _log("oracle chain 0 of cfg 4:", R, "rounds; states taken at a =", picks)
    for shift in range(3):
        a_host = np.array([picks[(c + shift) % 3] for c in range(B)], np.int32)
        ya = np.stack([y[a] for a in a_host]).astype(np.float32)
        _full_size_round(4, sampled=[0, 1, 2], states=(a_host, ya))
