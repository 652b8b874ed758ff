"""The arithmetic behind the work the mixture denoiser's verify call leaves out, checked on the CPU (numpy only; no
product or oracle code).

Four facts the bit-identity of the screened path rests on:
 * the int8 screening product's error bound: with x ~ sx qx and mu ~ sg qm (nearest integers in [-127, 127]),
   |sx sg <qx, qm> - <x, mu>| <= (sg / 2) |x|_1 + (sx / 2) |sg qm|_1;
 * the bounds U, L the decision is taken with really bracket the logits of a group, so that a tile declared dead
   holds only logits more than the zero gap below their rows' maxima -- and such logits get weights of exactly 0.0f:
   the kernels cut a weight off below 2^-gap of its row's largest, which moves a result by less than fp32 rounding does;
 * a row with one weight of 1.0 and zeros gets mu_b bit for bit from the split-operand accumulation: the three bf16
   pieces of an fp32 number add up exactly in the order the matrix cores add them;
 * the one-hot certificate: with e = x - s mu_b and a_n = |mu_n - mu_b|, logit_n - logit_b <= -(A/2) a_n^2 + B a_n
   + (A/2 - gamma') (|mu_n|^2 - |mu_b|^2) + log2 w_n - log2 w_b  (A = kappa' s, B = kappa' |e|), largest at the
   nearest neighbour of mu_b once that lies beyond the parabola's vertex, so a row that passes has all other logits
   more than the zero gap (plus what fp32 sums may be off by) below logit b.
"""
import numpy as np

from test_split_scheme import cut3

F = np.float32
LOG2E = F(1.4426950408889634)
ZERO_GAP = F(40.0)      # the kernels' zero gap: weights below 2^-40 of the row's largest are zero by definition


def quant(v):
    """The quantiser of the screening pass, in fp32 as the kernels run it: one scale for the array it is given."""
    v = np.asarray(v, dtype=F)
    mx = F(np.max(np.abs(v))) if v.size else F(0)
    s = F(mx / F(127)) if mx > 0 else F(1)
    inv = F(F(1) / s)
    q = np.clip(np.rint((v * inv).astype(F)), -127, 127).astype(np.int32)
    return s, q


def test_quantised_dot_product_is_within_its_bound():
    rng = np.random.default_rng(0)
    worst = 0.0
    for trial in range(200):
        d = int(rng.choice([128, 256, 1024, 2048]))
        heavy = trial % 3 == 0
        x = (rng.standard_t(2, d) if heavy else rng.standard_normal(d)).astype(F) * F(10.0 ** rng.uniform(-3, 3))
        mus = (2.0 * rng.standard_normal((64, d))).astype(F)               # one group of components: one scale
        if trial % 5 == 0:
            x[rng.integers(0, d, d // 2)] = 0
        sx, qx = quant(x)
        sg, qm = quant(mus)
        approx = float(sx) * float(sg) * (qm.astype(np.int64) @ qx.astype(np.int64))      # exact integer sums
        exact = mus.astype(np.float64) @ x.astype(np.float64)
        bound = 0.5 * float(sg) * np.abs(x.astype(np.float64)).sum() + \
            0.5 * float(sx) * float(sg) * np.abs(qm).sum(axis=1).astype(np.float64)
        # 1.001: the quantiser divides in fp32, so a value can land 127 * 2^-23 of a step off the nearest integer
        assert np.all(np.abs(approx - exact) <= 1.001 * bound)
        worst = max(worst, float(np.max(np.abs(approx - exact) / bound)))
    assert 0.05 < worst <= 1.001          # the bound is not vacuous either


def _logits_exact(x, mus, kappa, gamma, logw):
    """kappa' <x, mu_n> - gamma' |mu_n|^2 + log2 w_n in double (kappa', gamma' already in base-2 units)."""
    return kappa * (mus.astype(np.float64) @ x.astype(np.float64)) - gamma * (mus.astype(np.float64) ** 2).sum(1) + logw


def test_group_bounds_bracket_the_logits_and_dead_means_zero_weight():
    """The decision of the screening pass, re-derived here in fp32 from the quantities it is given, against logits in
    double: no logit of a group above U, the largest above L, and whatever lies more than the gap below a row's
    largest L -- everything the pass may leave out -- is a weight of exactly 0.0f."""
    rng = np.random.default_rng(1)
    d, n_groups, per = 256, 12, 64
    left_out = 0
    for trial in range(60):
        mus = (2.0 * rng.standard_normal((n_groups * per, d))).astype(F)
        logw = (LOG2E * np.log(rng.dirichlet(np.ones(n_groups * per)))).astype(F)
        ab = float(rng.uniform(0.02, 0.999))
        V = ab * 0.25 + 1 - ab
        kappa, gamma = F(LOG2E * F(np.sqrt(ab) / V)), F(LOG2E * F(ab / (2 * V)))
        b = int(rng.integers(0, n_groups * per))
        x = (np.sqrt(ab) * (mus[b] + 0.5 * rng.standard_normal(d)) + np.sqrt(1 - ab) * rng.standard_normal(d)).astype(F)
        sx, qx = quant(x)
        l1x = F(np.abs(x).sum(dtype=F) * F(1 + 1e-5))
        exact = _logits_exact(x, mus, float(kappa), float(gamma), logw.astype(np.float64))
        musq = (mus.astype(F) ** 2).sum(1, dtype=F)
        U, L = np.empty(n_groups, F), np.empty(n_groups, F)
        for g in range(n_groups):
            sl = slice(g * per, (g + 1) * per)
            sg, qm = quant(mus[sl])
            imax = int((qm.astype(np.int64) @ qx.astype(np.int64)).max())
            l1m = F(F(sg) * F(np.abs(qm).sum(axis=1).max()) * F(1 + 1e-6))
            base = F(F(kappa * sx) * sg * F(imax))
            ea = F(F(0.5) * F(1.001) * F(1.05) * kappa * l1x)
            eb = F(F(0.5) * F(1.001) * kappa * sx)
            e = F(ea * sg + (eb * l1m + F(0.5))) + F(1e-6) * (abs(base) + gamma * musq[sl].max())
            U[g] = base - gamma * musq[sl].min() + logw[sl].max() + e
            L[g] = base - gamma * musq[sl].max() + logw[sl].min() - e
            n_star = int(np.argmax(qm.astype(np.int64) @ qx.astype(np.int64)))
            assert exact[sl].max() <= U[g] and exact[sl][n_star] >= L[g]
        row_max = exact.max()
        assert L.max() <= row_max
        dead = U < L.max() - ZERO_GAP
        for g in np.nonzero(dead)[0]:
            sl = slice(g * per, (g + 1) * per)
            # as the second GEMM forms the weights: zero below lo = fl(row maximum - gap), else exp2 of an fp32 difference
            lo = F(F(row_max) - ZERO_GAP)
            lg = exact[sl].astype(F)
            wts = np.where(lg < lo, F(0), np.exp2((lg - F(row_max)).astype(F), dtype=F))
            assert np.all(exact[sl] < row_max - float(ZERO_GAP)) and np.all(wts == 0)
            left_out += 1
    assert left_out > 100                    # the test does leave groups out


def test_weights_below_the_gap_move_a_result_by_less_than_fp32_rounding():
    """The kernels take a softmax weight below 2^-gap of its row's largest as zero.  With w_max = 1 the sum of the
    weights is at least 1, the weights cut off add up to less than C 2^-gap, and the posterior mean moves by less than
    2 C 2^-gap max |mu|: for C = 4096 that is 2^-27, an eighth of fp32's unit roundoff.  Brute force in double on logits
    with gaps of every size around the cut."""
    rng = np.random.default_rng(5)
    gap = float(ZERO_GAP)
    worst = 0.0
    for trial in range(200):
        C, d = int(rng.integers(2, 600)), int(rng.integers(1, 9))
        mu = rng.standard_normal((C, d)) * rng.choice([0.1, 2.0, 50.0])
        logits = -rng.exponential(rng.choice([1.0, 15.0, 40.0, 100.0]), C)     # base-2 units, largest near 0
        logits[rng.integers(0, C)] = 0.0
        logits[rng.integers(0, C, 3)] = -gap + rng.uniform(-1e-3, 1e-3, 3)      # some right at the cut
        w = np.exp2(logits - logits.max())
        exact = (w[:, None] * mu).sum(0) / w.sum()
        wc = np.where(logits < logits.max() - gap, 0.0, w)
        cut = (wc[:, None] * mu).sum(0) / wc.sum()
        bound = 2.0 * C * 2.0 ** -gap * np.abs(mu).max()
        assert np.abs(cut - exact).max() <= bound
        worst = max(worst, np.abs(cut - exact).max() / np.abs(mu).max())
    assert 2.0 * 4096 * 2.0 ** -gap <= 2.0 ** -27 and worst <= 2.0 ** -27
    assert np.exp2(F(0.0), dtype=F) == 1


def test_one_hot_row_gives_the_mean_bit_for_bit():
    """Weights (1.0, 0, 0, ...): the six products per element reduce to 1.0 * mu1, 1.0 * mu2, 1.0 * mu3 (the pieces of
    1.0 are 1.0, 0, 0), added in that order to an accumulator that starts at +0: every partial sum is exact."""
    rng = np.random.default_rng(2)
    mu = np.concatenate([(2.0 * rng.standard_normal(100000)).astype(F),
                         np.array([0.0, 1.0, -1.0, 3e38, 1e-30, 1 + 2.0 ** -23, -(1 + 2.0 ** -22)], dtype=F)])
    m1, m2, m3 = cut3(mu)
    a1, a2, a3 = cut3(np.ones_like(mu))
    assert np.all(a1 == 1) and np.all(a2 == 0) and np.all(a3 == 0)
    acc = np.zeros_like(mu)
    for pa, pb in ((a1, m1), (a1, m2), (a2, m1), (a2, m2), (a1, m3), (a3, m1)):     # the kernel's order of plane pairs
        acc = (acc + (pa * pb).astype(F)).astype(F)
    assert np.array_equal(acc.view(np.uint32), (mu + F(0)).view(np.uint32))
    # and the epilogue: scale = c_m' / 1.0 is c_m', out = fma(c_x', x, scale * acc) -- the same expression either way
    assert F(0.37) / F(1.0) == F(0.37)


def test_onehot_certificate_bounds_every_other_logit():
    """The one-hot certificate, re-derived in fp32 as its kernel evaluates it (nearest-neighbour distance rounded
    down, s = <x, mu_b> / |mu_b|^2, the parabola beyond its vertex, the margin for what computed logits may be off
    by), against the logit differences in double: the bound really is one, a certified row is one-hot with room to
    spare for the fp32 sums of the exact path, rows late in the chain do get certified, and a wrong candidate never is."""
    rng = np.random.default_rng(3)
    d, C = 256, 384
    means = (2.0 * rng.standard_normal((C, d))).astype(F)
    means[7] = means[3] + F(0.05) * rng.standard_normal(d).astype(F)     # two components close together
    logw2 = (LOG2E * np.log(rng.dirichlet(np.ones(C))).astype(F)).astype(F)
    m64 = means.astype(np.float64)
    musq = (means ** 2).sum(1, dtype=F)
    dist = np.sqrt(((m64[None, :, :] - m64[:, None, :]) ** 2).sum(2))
    np.fill_diagonal(dist, np.inf)
    a_min = (np.nextafter(dist.min(1).astype(F), F(0)) * F(1 - 1e-6)).astype(F)    # rounded down
    mumax = F(np.sqrt(musq.max()) * F(1.001))
    qmax, qmin = musq.max(), musq.min()
    bmax, babs = logw2.max(), np.abs(logw2).max()
    certified = wrong_certified = 0
    for trial in range(400):
        ab = float(rng.uniform(0.2, 0.9995))
        V = ab * 0.25 + 1 - ab
        c1, c2 = F(LOG2E * F(np.sqrt(ab) / V)), F(LOG2E * F(ab / (2 * V)))
        b = 3 if trial % 50 == 0 else int(rng.integers(0, C))
        x = (np.sqrt(ab) * (means[b] + 0.5 * rng.standard_normal(d)) + np.sqrt(1 - ab) * rng.standard_normal(d)).astype(F)
        # the logits as exact arithmetic on what the kernels are given (musq and log2 w as fp32 numbers)
        exact = float(c1) * (m64 @ x.astype(np.float64)) - float(c2) * musq.astype(np.float64) + logw2.astype(np.float64)
        for cand in (b, (b + 1) % C):
            s = F(np.dot(x, means[cand]) / musq[cand])
            e = (x - s * means[cand]).astype(F)
            e_up = F(np.sqrt(np.dot(e, e)) * F(1 + 2.0 ** -10))
            x_up = F(np.sqrt(np.dot(x, x)) * F(1 + 2.0 ** -10))
            A, B = F(c1 * s), F(c1 * e_up)
            half, am, qb = F(0.5) * A, a_min[cand], musq[cand]
            f = F(am * (B - half * am))
            beyond = bool(am * A >= B)
            dq = F(half - c2)
            qterm = F(dq * ((qmax if dq >= 0 else qmin) - qb))
            bterm = F(bmax - logw2[cand])
            mag = (am * B + half * am * am) + abs(qterm) + (babs + abs(logw2[cand])) + c2 * qmax
            margin = F(c1 * x_up * mumax * F(2.0 ** -9 + 1e-5) + ((c2 + abs(dq)) * qmax * F(2.0 ** -12) + (F(1e-5) * mag + F(1))))
            bound = F(f + qterm + bterm)
            others = np.arange(C) != cand
            gap = exact - exact[cand]
            if s >= 0 and beyond:
                # Cauchy-Schwarz and the parabola, whatever the candidate: every exact difference lies below the
                # bound (musq against |mu|^2 and this fp32 evaluation against double: inside the margin less the
                # part that is for the exact path's sums)
                assert np.all(gap[others] <= float(bound) + float((c2 + abs(dq)) * qmax * F(2.0 ** -12)) + 1e-5 * float(mag))
            ok = bool(s >= 0 and beyond and bound + (ZERO_GAP + margin) < 0)
            if ok:
                # one-hot, with room for two fp32 split-operand sums (2^-10 |x| |mu| each) on top of the zero gap
                room = float(c1) * 2.0 ** -9 * float(x_up) * float(mumax)
                assert np.all(gap[others] < -float(ZERO_GAP) - room)
                wts = np.exp2((exact[others] - exact[cand]).astype(F), dtype=F)
                assert np.all(wts == 0)
            certified += ok and cand == b
            wrong_certified += ok and cand != b
            assert not (ok and cand in (3, 7))          # their nearest neighbour is too close at any noise level here
    assert certified > 60 and wrong_certified == 0
