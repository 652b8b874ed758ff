"""Philox4x32-10 counter-based generator, uniforms and normals (oracle side).

Test infrastructure; never imported by the product path.

The generator is the one defined by Salmon, Moraes, Dror and Shaw, "Parallel
random numbers: as easy as 1, 2, 3" (SC'11): four 32-bit counter words, two
32-bit key words, ten rounds.  Alg. 1 of the ASD paper draws (u_1..u_K) and
(xi_1..xi_K) once and indexes them by *step*; a counter-based generator makes
that indexing literal: the counter is (block, step, chain, stream) and the key
is the 64-bit seed, so the value attached to a step never depends on the round
in which it is consumed.

Counter layout (shared by convention with the device code, not by code):
    ctr[0] = block   index of a group of four consecutive coordinates
    ctr[1] = step    i in 0..K (0 = the initial state y_0, i>=1 = xi_i / u_i)
    ctr[2] = chain   chain id
    ctr[3] = stream  0: normals xi, 1: uniforms u
    key    = (seed mod 2^32, seed div 2^32)
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_SH = np.uint64(32)

STREAM_XI = 0
STREAM_U = 1


def philox4x32_10(ctr, key):
    """Ten Philox rounds.  ctr: integer array [..., 4]; key: two 32-bit ints.

    Returns uint32 array [..., 4].  One round multiplies words 0 and 2 by the
    two round constants, and recombines high/low halves with words 1 and 3 and
    the key; the key is bumped by the Weyl constants between rounds.
    """
    ctr = np.asarray(ctr)
    c0 = ctr[..., 0].astype(np.uint64)
    c1 = ctr[..., 1].astype(np.uint64)
    c2 = ctr[..., 2].astype(np.uint64)
    c3 = ctr[..., 3].astype(np.uint64)
    k0 = int(key[0]) & 0xFFFFFFFF
    k1 = int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH, p0 & _MASK
        hi1, lo1 = p1 >> _SH, p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0)), lo1, (hi0 ^ c3 ^ np.uint64(k1)), lo0
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def seed_key(seed):
    seed = int(seed)
    return (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)


def word_to_uniform(w):
    """Top 23 bits of a word, centred: ((w >> 9) + 1/2) * 2^-23, in (0, 1).

    Exactly representable in fp32, never 0 or 1.
    """
    return ((np.asarray(w, dtype=np.uint32) >> np.uint32(9)).astype(np.float64) + 0.5) * 2.0 ** -23


def _box_muller(ua, ub):
    r = np.sqrt(-2.0 * np.log(ua))
    ang = 2.0 * np.pi * ub
    return r * np.cos(ang), r * np.sin(ang)


def normals(seed, chain, steps, d):
    """Standard normals xi[step, 0:d] for the given chain (fp64).

    steps: iterable of step indices.  Each Philox block gives four words
    (w0..w3); coordinates 4*blk+0, +1 come from Box-Muller on (w0, w1) as
    (r cos, r sin), coordinates +2, +3 from (w2, w3).
    """
    steps = np.asarray(list(steps), dtype=np.int64)
    nblk = (d + 3) // 4
    ctr = np.zeros((len(steps), nblk, 4), dtype=np.uint64)
    ctr[..., 0] = np.arange(nblk, dtype=np.uint64)[None, :]
    ctr[..., 1] = steps[:, None].astype(np.uint64)
    ctr[..., 2] = np.uint64(chain)
    ctr[..., 3] = np.uint64(STREAM_XI)
    w = philox4x32_10(ctr, seed_key(seed))
    u = word_to_uniform(w)
    n0, n1 = _box_muller(u[..., 0], u[..., 1])
    n2, n3 = _box_muller(u[..., 2], u[..., 3])
    out = np.stack([n0, n1, n2, n3], axis=-1).reshape(len(steps), nblk * 4)
    return out[:, :d]


def uniforms(seed, chain, steps):
    """Uniforms u[step] in (0,1) for the given chain (word 0 of block 0)."""
    steps = np.asarray(list(steps), dtype=np.int64)
    ctr = np.zeros((len(steps), 4), dtype=np.uint64)
    ctr[:, 1] = steps.astype(np.uint64)
    ctr[:, 2] = np.uint64(chain)
    ctr[:, 3] = np.uint64(STREAM_U)
    w = philox4x32_10(ctr, seed_key(seed))
    return word_to_uniform(w[:, 0])
