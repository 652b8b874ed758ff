"""CPU oracle for Autospeculative Decoding (ASD) of DDPM sampling.

TEST INFRASTRUCTURE ONLY.  This package is the plain, slow, fp64 statement of
what the hot path computes.  Only ``tests/``, ``__graft_entry__.smoke()`` and
the ``cpu_baseline`` leg of ``bench.py`` may import it.  It shares no code with
the HIP library: every formula, table builder and random-number routine is
written out here a second time, from the paper, in numpy.

Modules
-------
philox     counter-based random numbers (Philox4x32-10; Salmon et al., SC'11)
schedule   DDPM linear-beta tables in x0-prediction form (Remark after Alg. 3)
           and the map to Stochastic Localization time (Sec. 2.1, Thm. 1)
denoisers  Gaussian-mixture posterior mean (Eq. sl-defn specialised) and the
           residual MLP with bf16 rounding points
grs        Gaussian Rejection Sampler (Alg. 3)
asd        sequential chain (Eq. euler-sde) and ASD (Alg. 1 with Alg. 2)

Parity status: every function is pinned by tests under ``tests/`` marked
"not gpu", except the MLP forward pass, whose definition is not in the paper:
it is pinned only by special cases (hand-computed example, zero/identity
weights) -- "parity unpinned" with respect to the paper.
"""
