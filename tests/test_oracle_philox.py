"""Pins for the oracle's random numbers (Alg. 1: u_{1:K}, xi_{1:K} drawn once,
indexed by step)."""
import os

import numpy as np
from scipy import stats

from oracle import philox

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_known_answers():
    n = 0
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        out = philox.philox4x32_10(np.array(w[0:4], dtype=np.uint64), w[4:6])
        assert [int(x) for x in out] == w[6:10]
        n += 1
    assert n == 3


def test_uniform_is_open_interval_and_fp32_exact():
    w = np.array([0, 1, 511, 512, 0xFFFFFFFF, 0x80000000], dtype=np.uint32)
    u = philox.word_to_uniform(w)
    assert u.min() > 0.0 and u.max() < 1.0
    assert np.all(u.astype(np.float32).astype(np.float64) == u)
    assert u[0] == 2.0 ** -24 and u[4] == 1.0 - 2.0 ** -24
    assert u[0] == u[1] == u[2] and u[3] > u[2]          # low 9 bits unused


def test_uniform_and_normal_laws():
    K, d = 4000, 8
    u = np.concatenate([philox.uniforms(3, c, range(1, K + 1)) for c in range(4)])
    assert stats.kstest(u, "uniform").pvalue > 1e-3
    x = philox.normals(3, 0, range(K + 1), d).ravel()
    assert stats.kstest(x, "norm").pvalue > 1e-3
    assert abs(x.mean()) < 4 / np.sqrt(x.size)
    assert abs(x.var() - 1.0) < 4 * np.sqrt(2.0 / x.size)
    # coordinates of one draw are uncorrelated
    X = philox.normals(5, 1, range(1, 20001), 4)
    c = np.corrcoef(X.T)
    assert np.max(np.abs(c - np.eye(4))) < 0.03


def test_step_indexing_not_round_indexing():
    """A step's draw depends on (seed, chain, step) only; any subset of steps or
    chains reproduces (what lets a chain subset be checked in isolation)."""
    a = philox.normals(11, 2, range(0, 50), 10)
    b = philox.normals(11, 2, [7, 49], 10)
    assert np.array_equal(a[[7, 49]], b)
    assert not np.array_equal(philox.normals(11, 3, [7], 10), b[:1])
    assert not np.array_equal(philox.normals(12, 2, [7], 10), b[:1])
    # d that is not a multiple of four is a prefix of the padded draw
    assert np.array_equal(philox.normals(11, 2, [7], 12)[:, :10], b[:1])
    ua = philox.uniforms(11, 2, range(1, 50))
    assert np.array_equal(ua[[6]], philox.uniforms(11, 2, [7]))
    # 64-bit seeds use both key words
    assert not np.array_equal(philox.uniforms(1 << 32, 0, [1]), philox.uniforms(0, 0, [1]))
