"""The arithmetic behind the split-operand GEMM, checked on the CPU (numpy only; no product or oracle code).

The kernel cuts every fp32 operand into three bf16 pieces by truncation and replaces a*b by the six
products whose weight is at least 2^-16 of it.  These tests pin the two facts the kernel's accuracy
rests on: the cut is exact, and the six-term product is accurate to a few units of fp32 rounding.

Where the shape allows, the kernel takes two fp16 pieces per operand instead (11-bit significands, rounded to
nearest, operands scaled by powers of two into fp16's upper range) and three products: the same accuracy from half
the matrix instructions.  Pinned likewise: the two pieces carry 22 bits, and the three-term product is within the
six-term one's bound.
"""
import numpy as np


def cut3(x):
    """x (float32 array) -> three float32 arrays whose low 16 bits are zero (bf16-representable), by truncation:
    the top 16 bits of x, the top 16 bits of the remainder, the rest."""
    x = np.asarray(x, dtype=np.float32)
    top = lambda v: (v.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    x1 = top(x)
    r = (x - x1).astype(np.float32)
    x2 = top(r)
    x3 = (r - x2).astype(np.float32)
    return x1, x2, x3


def _samples(rng, n):
    mag = np.exp(rng.uniform(np.log(1e-6), np.log(1e6), n))
    x = (mag * rng.choice([-1.0, 1.0], n)).astype(np.float32)
    x[:8] = [0.0, -0.0, 1.0, -1.0, 3.0e38, -3.0e38, 1.17549435e-38, 1.0 + 2.0 ** -23]
    return x


def test_three_bf16_pieces_are_exact():
    rng = np.random.default_rng(0)
    x = _samples(rng, 200000)
    x1, x2, x3 = cut3(x)
    for p in (x1, x2, x3):
        assert np.all((p.view(np.uint32) & np.uint32(0xFFFF)) == 0)          # each piece is a bf16 number
    # exact: the pieces add up to x in any order, evaluated in double
    assert np.array_equal(x1.astype(np.float64) + x2.astype(np.float64) + x3.astype(np.float64), x.astype(np.float64))
    # same sign, decreasing by at least 2^-8 each
    nz = x != 0
    assert np.all(np.abs(x2[nz]) <= np.abs(x1[nz]) * 2.0 ** -7)
    assert np.all(np.abs(x3[nz]) <= np.abs(x1[nz]) * 2.0 ** -15)


def test_six_products_are_within_a_few_fp32_roundings():
    rng = np.random.default_rng(1)
    a, b = _samples(rng, 100000)[8:], _samples(rng, 100000)[8:][::-1].copy()
    a1, a2, a3 = (p.astype(np.float64) for p in cut3(a))
    b1, b2, b3 = (p.astype(np.float64) for p in cut3(b))
    six = a1 * b1 + a1 * b2 + a2 * b1 + a2 * b2 + a1 * b3 + a3 * b1           # each product is exact in fp32
    exact = a.astype(np.float64) * b.astype(np.float64)
    err = np.abs(six - exact)
    # what is dropped is a2 b3 + a3 b2 + a3 b3, with |x2| < 2^-7 |x1| and |x3| < 2^-15 |x1|: below 2^-21 |a b| always,
    # 2^-23 |a b| on average (an fp32 multiply rounds by up to 2^-24 |a b|)
    assert np.all(err <= 1.01 * 2.0 ** -21 * np.abs(exact))
    assert np.mean(err / np.abs(exact)) <= 1.3 * 2.0 ** -23
    # a dot product accumulated from these terms is within fp32 rounding of the exact one
    K = 4096
    x, y = rng.standard_normal(K).astype(np.float32), rng.standard_normal(K).astype(np.float32)
    xs, ys = [p.astype(np.float64) for p in cut3(x)], [p.astype(np.float64) for p in cut3(y)]
    dot6 = sum(np.dot(xs[i], ys[j]) for i, j in ((0, 0), (0, 1), (1, 0), (1, 1), (0, 2), (2, 0)))
    ref = np.dot(x.astype(np.float64), y.astype(np.float64))
    assert abs(dot6 - ref) <= 2.0 ** -24 * np.sum(np.abs(x.astype(np.float64) * y.astype(np.float64)))
    # leaving out the 2^-16 terms would not be: the two-piece, three-product variant is ~2^8 times worse
    dot3 = np.dot(xs[0], ys[0]) + np.dot(xs[0], ys[1]) + np.dot(xs[1], ys[0])
    assert abs(dot3 - ref) > 20 * abs(dot6 - ref)


def cut2(x, scale):
    """x (float32 array), scale (a power of two) -> the two fp16 pieces of scale * x as float32 arrays: the nearest
    fp16, and the nearest fp16 of the remainder (which is exact in fp32)."""
    xs = (np.asarray(x, dtype=np.float32) * np.float32(scale)).astype(np.float32)
    x1 = xs.astype(np.float16).astype(np.float32)
    x2 = (xs - x1).astype(np.float32).astype(np.float16).astype(np.float32)
    return x1, x2


def fp16_scale(mx):
    """The power of two that brings a largest magnitude into [2^14, 2^15) (fp16's largest finite number is 65504)."""
    return 2.0 ** (15 - (int(np.floor(np.log2(mx))) + 1))


def test_two_fp16_pieces_carry_22_bits():
    rng = np.random.default_rng(4)
    for row_max in (1e-6, 0.03, 4.0, 900.0, 3e9):
        x = (row_max * rng.uniform(-1, 1, 50000) * np.exp(rng.uniform(np.log(1e-7), 0.0, 50000))).astype(np.float32)
        x[0] = row_max                                               # the row's largest element fixes the scale
        s = fp16_scale(float(np.abs(x).max()))
        assert 2.0 ** 14 <= float(np.abs(x).max()) * s < 2.0 ** 15
        x1, x2 = cut2(x, s)
        assert np.all(np.isfinite(x1)) and np.all(np.abs(x1) <= 32768.0)
        rep = (x1.astype(np.float64) + x2.astype(np.float64)) / s
        err = np.abs(rep - x.astype(np.float64))
        # 2^-22 of the element while its second piece is a normal fp16 number; below that the pieces sit on fp16's
        # subnormal grid (spacing 2^-24 in scaled units), i.e. 2^-25 / 2^14 = 2^-39 of the row's largest element
        assert np.all(err <= 2.0 ** -22 * np.abs(x.astype(np.float64)) + 2.0 ** -39 * float(np.abs(x).max()))
        # the sum of the two pieces is itself an fp32 number: what a weight of 1.0 reproduces bit for bit
        both = (x1 + x2).astype(np.float32)
        assert np.array_equal(both.astype(np.float64), x1.astype(np.float64) + x2.astype(np.float64))


def test_three_fp16_products_match_the_six_bf16_ones():
    rng = np.random.default_rng(5)
    n = 100000
    a = (rng.standard_normal(n) * np.exp(rng.uniform(-3, 3, n))).astype(np.float32)
    b = (rng.standard_normal(n) * np.exp(rng.uniform(-3, 3, n))).astype(np.float32)
    sa, sb = fp16_scale(float(np.abs(a).max())), fp16_scale(float(np.abs(b).max()))
    a1, a2 = (p.astype(np.float64) for p in cut2(a, sa))
    b1, b2 = (p.astype(np.float64) for p in cut2(b, sb))
    three = (a1 * b1 + a1 * b2 + a2 * b1) / (sa * sb)                 # each product is exact in fp32
    exact = a.astype(np.float64) * b.astype(np.float64)
    big = (np.abs(a) > 2.0 ** -10 * np.abs(a).max()) & (np.abs(b) > 2.0 ** -10 * np.abs(b).max())   # second pieces normal
    err = np.abs(three - exact)
    # dropped: a2 b2 (2^-22 |a b| at most) and what the pieces miss of a and of b (2^-22 each): 3 * 2^-22 at most,
    # about 2^-23 on average -- the six-product bf16 scheme's figures are 2^-21 and 2^-23
    assert np.all(err[big] <= 3.03 * 2.0 ** -22 * np.abs(exact[big]))
    assert np.mean(err[big] / np.abs(exact[big])) <= 1.3 * 2.0 ** -23
    # a dot product accumulated from these terms is within fp32 rounding of the exact one, as with six bf16 products
    K = 4096
    x, y = rng.standard_normal(K).astype(np.float32), (2.0 * rng.standard_normal(K)).astype(np.float32)
    sx, sy = fp16_scale(float(np.abs(x).max())), fp16_scale(float(np.abs(y).max()))
    xs, ys = [p.astype(np.float64) for p in cut2(x, sx)], [p.astype(np.float64) for p in cut2(y, sy)]
    dot3 = (np.dot(xs[0], ys[0]) + np.dot(xs[0], ys[1]) + np.dot(xs[1], ys[0])) / (sx * sy)
    ref = np.dot(x.astype(np.float64), y.astype(np.float64))
    assert abs(dot3 - ref) <= 2.0 ** -24 * np.sum(np.abs(x.astype(np.float64) * y.astype(np.float64)))
    # without the scaling small rows would lose their second pieces to fp16's subnormal grid
    tiny = (1e-3 * x).astype(np.float32)
    t1, t2 = (p.astype(np.float64) for p in cut2(tiny, 1.0))
    u1, u2 = (p.astype(np.float64) for p in cut2(tiny, fp16_scale(float(np.abs(tiny).max()))))
    s_t = fp16_scale(float(np.abs(tiny).max()))
    assert np.abs(t1 + t2 - tiny).max() > 30 * np.abs((u1 + u2) / s_t - tiny).max()


def test_one_hot_row_gives_the_two_term_mean_bit_for_bit():
    """fp16 terms: a weight of 1.0 enters as 2^15 = (32768, 0); the three products per element are 32768 m1,
    32768 m2 and 0 m1, added to an accumulator that starts at +0: exact, so the row's result is (m1 + m2) / scale --
    the means as gmm_means22_kernel stores them, not the caller's."""
    rng = np.random.default_rng(6)
    mu = np.concatenate([(2.0 * rng.standard_normal(100000)).astype(np.float32),
                         np.array([0.0, 1.0, -1.0, 9.99, 1e-9, 1 + 2.0 ** -23, -(1 + 2.0 ** -12)], dtype=np.float32)])
    s = fp16_scale(float(np.abs(mu).max()))
    m1, m2 = cut2(mu, s)
    w1, w2 = cut2(np.ones_like(mu), 32768.0)
    assert np.all(w1 == 32768.0) and np.all(w2 == 0)
    acc = np.zeros_like(mu)
    for pa, pb in ((w1, m1), (w1, m2), (w2, m1)):
        acc = (acc + (pa * pb).astype(np.float32)).astype(np.float32)
    mu22 = ((m1 + m2).astype(np.float32) / np.float32(s)).astype(np.float32)
    got = (acc / np.float32(32768.0 * s)).astype(np.float32)
    assert np.array_equal(got.view(np.uint32), (mu22 + np.float32(0)).view(np.uint32))
    assert np.all(np.abs(mu22.astype(np.float64) - mu.astype(np.float64)) <= 2.0 ** -22 * np.abs(mu) + 2.0 ** -39 * np.abs(mu).max())
