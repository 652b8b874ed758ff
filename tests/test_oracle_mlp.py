"""Pins for the MLP denoiser of the oracle.  Its definition is not in the
paper ("parity unpinned"): only special cases and a hand-computed example."""
import numpy as np
import pytest
import torch

import asd_workloads as W
from oracle import denoisers


def test_bf16_rounding_matches_library_conversion():
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, 5000),
                        [1.00390625, 1.01171875, 0.0, -0.0, 3.0e38]])   # two exact ties
    ref = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(denoisers.round_to_bf16(a), ref)
    bits = W.f32_to_bf16_bits(a.astype(np.float32))
    np.testing.assert_array_equal(denoisers.bf16_bits_to_f64(bits), ref)


def _params(w_in, w_blk, w_out, temb):
    f = W.f32_to_bf16_bits
    return dict(w_in=f(w_in), w_blk=f(w_blk), w_out=f(w_out), temb=f(temb),
                b_in=np.zeros(w_in.shape[0], np.float32), b_blk=np.zeros(w_blk.shape[:2], np.float32),
                b_out=np.zeros(w_out.shape[0], np.float32))


def test_hand_computed_two_wide_example():
    # d=1, E=1, width=2, one block; all values exactly representable in bf16.
    w_in = np.array([[1.0, 0.5], [-2.0, 1.0]], np.float32)        # rows: out, cols: [x, temb]
    w_blk = np.array([[[1.0, 0.0], [0.5, 0.5]]], np.float32)
    w_out = np.array([[2.0, -1.0]], np.float32)
    temb = np.array([[0.0], [4.0], [-2.0]], np.float32)            # tau = 0,1,2
    mlp = denoisers.MLPOracle(_params(w_in, w_blk, w_out, temb))
    x, tau = 0.5, 2
    h = np.array([1.0 * x + 0.5 * -2.0, -2.0 * x + 1.0 * -2.0])   # [-0.5, -3.0]
    zlin = np.array([h[0], 0.5 * h[0] + 0.5 * h[1]])              # [-0.5, -1.75]
    h1 = h + zlin / (1 + np.exp(-zlin))
    h1r = denoisers.round_to_bf16(h1)
    want = 2.0 * h1r[0] - 1.0 * h1r[1]
    got = mlp([[x]], [tau])[0, 0]
    assert abs(got - want) < 1e-15
    p = _params(w_in, w_blk, w_out, temb)
    p["b_in"] = np.array([0.25, -1.0], np.float32)
    p["b_out"] = np.array([3.0], np.float32)
    p["w_blk"] = np.zeros_like(p["w_blk"])
    # zero block weights: SiLU(0) = 0, the block is the identity
    got = denoisers.MLPOracle(p)([[x]], [1])[0, 0]
    h = np.array([1.0 * x + 0.5 * 4.0 + 0.25, -2.0 * x + 4.0 - 1.0])
    assert abs(got - (2 * h[0] - h[1] + 3.0)) < 1e-15


def test_two_term_activation_rounding():
    """An activation as the sum of two bf16 numbers: both terms are bf16 values, the sum is within 2^-16 of the
    value (8 bits from each term), values of at most 16 significant bits survive exactly, and it agrees with
    the same construction done with the library's own conversions."""
    rng = np.random.default_rng(5)
    a = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-5, 5, 4000), [0.0, 1.0 + 2.0 ** -10, 40503.0]])
    a32 = a.astype(np.float32).astype(np.float64)
    two = denoisers.round_to_bf16_terms(a, 2)
    hi = denoisers.round_to_bf16(a)
    lo = two - hi
    np.testing.assert_array_equal(denoisers.round_to_bf16(lo), lo)            # the second term is a bf16 number
    assert np.all(np.abs(two - a32) <= 2.0 ** -16 * np.abs(a32))
    assert np.all(np.abs(hi - a32) <= 2.0 ** -8 * np.abs(a32)) and np.any(np.abs(hi - a32) > 2.0 ** -11 * np.abs(a32))
    assert two[-2] == 1.0 + 2.0 ** -10 and hi[-2] == 1.0 and two[-1] == 40503.0 and hi[-1] != 40503.0
    t = torch.from_numpy(a.astype(np.float32))
    t_hi = t.to(torch.bfloat16).to(torch.float32)
    t_lo = (t - t_hi).to(torch.bfloat16).to(torch.float32)
    np.testing.assert_array_equal(two, t_hi.to(torch.float64).numpy() + t_lo.to(torch.float64).numpy())
    np.testing.assert_array_equal(denoisers.round_to_bf16_terms(a, 1), hi)
    with pytest.raises(ValueError):
        denoisers.round_to_bf16_terms(a, 3)


def test_two_term_network_is_the_unrounded_network_to_sixteen_bits():
    """With exact activations (no rounding at all) as the yardstick: one-term activations sit at the 2^-9
    level of the output scale, two-term ones a hundred times closer."""
    p1 = W.mlp_params(d=24, E=8, width=256, n_blocks=4, K=10, model_seed=4, out_clip=0.0, act_terms=1)
    p2 = dict(p1, act_terms=2)
    rng = np.random.default_rng(2)
    x = rng.standard_normal((16, 24)).astype(np.float32).astype(np.float64)
    tau = rng.integers(1, 11, 16)
    f = denoisers.bf16_bits_to_f64
    h = np.concatenate([x, f(p1["temb"])[tau]], axis=1) @ f(p1["w_in"]).T
    for l in range(4):
        h = h + denoisers.silu(h @ f(p1["w_blk"])[l].T)
    exact = h @ f(p1["w_out"]).T
    scale = np.abs(exact).max()
    e1 = np.abs(denoisers.MLPOracle(p1)(x, tau) - exact).max() / scale
    e2 = np.abs(denoisers.MLPOracle(p2)(x, tau) - exact).max() / scale
    assert 2e-4 < e1 < 2e-2 and e2 < 5e-5 and e2 < e1 / 50, (e1, e2)


def test_rows_are_independent_and_rounding_points_matter():
    p = W.mlp_params(d=12, E=8, width=32, n_blocks=2, K=10, model_seed=3, act_terms=1)
    mlp = denoisers.MLPOracle(p)
    rng = np.random.default_rng(1)
    x = rng.standard_normal((6, 12))
    tau = np.array([1, 5, 10, 3, 3, 7])
    full = mlp(x, tau)
    for n in range(6):
        np.testing.assert_allclose(mlp(x[n:n + 1], tau[n:n + 1])[0], full[n], rtol=1e-13)
    # inputs that differ by less than half a bf16 ulp are the same to the network
    np.testing.assert_array_equal(mlp(np.full((1, 12), 1.0), [2]), mlp(np.full((1, 12), 1.0 + 2.0 ** -10), [2]))
    assert np.max(np.abs(full)) < 50 and np.std(full) > 0.05
    # ... but not to the network with two-term activations, which carries 16 bits of them
    mlp2 = denoisers.MLPOracle(dict(p, act_terms=2))
    assert not np.array_equal(mlp2(np.full((1, 12), 1.0), [2]), mlp2(np.full((1, 12), 1.0 + 2.0 ** -10), [2]))
    np.testing.assert_array_equal(mlp2(np.full((1, 12), 1.0 + 2.0 ** -10), [2]),
                                  mlp2(np.full((1, 12), 1.0 + 2.0 ** -10 + 2.0 ** -20), [2]))


def test_noise_prediction_is_the_affine_map_of_the_output():
    """predict_eps: x0hat = (x - sqrt(1 - abar) out) / sqrt(abar).  Pins: zero weights give
    out = b_out exactly, so x0hat = (x - sqrt(1 - abar) b) / sqrt(abar); and for any weights the
    result is that affine map of the x0-parametrised network's output (same rows, same time)."""
    import asd_workloads as W
    from oracle import denoisers, schedule
    K, d, E, width = 12, 8, 8, 16
    T = schedule.ddpm_tables(K)
    p = W.mlp_params(d, E, width, 2, K, model_seed=3, out_clip=0.0, predict_eps=True)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, d))
    tau = np.array([1, 4, 7, 12, 12])
    ab = T["abar"][tau][:, None]
    zero = dict(p, w_in=np.zeros_like(p["w_in"]), w_blk=np.zeros_like(p["w_blk"]), w_out=np.zeros_like(p["w_out"]),
                b_out=np.linspace(-1, 1, d).astype(np.float32))
    got = denoisers.MLPOracle(zero, abar=T["abar"])(x, tau)
    np.testing.assert_allclose(got, (x - np.sqrt(1 - ab) * zero["b_out"][None, :]) / np.sqrt(ab), rtol=1e-12)
    raw = denoisers.MLPOracle(dict(p, predict_eps=False))(x, tau)
    eps = denoisers.MLPOracle(p, abar=T["abar"])(x, tau)
    np.testing.assert_allclose(eps, (x - np.sqrt(1 - ab) * raw) / np.sqrt(ab), rtol=1e-12)
    clipped = denoisers.MLPOracle(dict(p, out_clip=1.0), abar=T["abar"])(x, tau)
    np.testing.assert_array_equal(clipped, np.clip(eps, -1.0, 1.0))
    with pytest.raises(ValueError):
        denoisers.MLPOracle(p)
