"""The arithmetic behind the split-operand GEMM, checked on the CPU (numpy only; no product or oracle code).

The kernel cuts every fp32 operand into three bf16 pieces by truncation and replaces a*b by the six
products whose weight is at least 2^-16 of it.  These tests pin the two facts the kernel's accuracy
rests on: the cut is exact, and the six-term product is accurate to a few units of fp32 rounding.
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
