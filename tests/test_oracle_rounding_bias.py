"""What the shared permutation of the correlated rounding (Section 3.3) does over SEVERAL hops.

One hop is unbiased by construction (uniform marginals, pinned in test_oracle_pins.py).  Along a
path of hops the input of hop i depends on how hop i-1 rounded, and the permutation ties the two
hops' uniforms together (worker i cannot get the interval worker i-1 has), so the estimate of a
multi-hop sum carries a small bias even with an ideally shuffled permutation: averaging R rounds
leaves err(R) = err(1) * (1/R + beta) with beta > 0.  These tests measure beta on the oracle's
core functions for rings of 8 and 64 workers, for the oracle's permutation law and for numpy's
uniformly random permutations on the same data, and check that
  - the law behaves like the ideal shuffle (same one-round error, same beta within noise),
  - beta stays below 0.03 (the bound the GPU statistics test uses),
  - a fixed-stride map  pi_i = (m i + c) mod n  -- a valid permutation with uniform marginals --
    has a beta several times larger: the measurement does tell a tied law from a shuffled one.
"""
import math

import numpy as np
import pytest

from oracle import dq_oracle as O

BETA_BOUND = 0.03


def ring_beta(n, wi, slots_of, R, n_sg, seed=0):
    """One chunk of n_sg super-groups travels a ring of n workers (compress, n-2 DAR hops, sink),
    R rounds with fresh random numbers.  slots_of(round, sg) -> the n workers' slots.
    Returns (one-round relative error, beta)."""
    rng = np.random.default_rng(seed)
    sc = 10.0 ** rng.uniform(-4, -2, n_sg)
    X = (rng.standard_normal((n, n_sg, 256)) * sc[None, :, None]).astype(np.float32)
    truth = X.astype(np.float64).sum(axis=0)
    orc = O.Oracle(n, seed=1)
    prng = np.random.default_rng(1000 + seed)
    acc = np.zeros_like(truth)
    e1 = 0.0
    for r in range(R):
        for j in range(n_sg):
            slots = slots_of(r, j)
            gam = prng.integers(0, 256, (n, 256), dtype=np.uint8)
            sb = prng.integers(0, 256, (n, 16), dtype=np.uint8)
            code, rG, sf = orc.encode_sg_core(wi, X[0, j], gam[0], sb[0], int(slots[0]))
            for w in range(1, n - 1):
                v = orc.decode_sg_core(wi, code, rG, sf, X[w, j])
                code, rG, sf = orc.encode_sg_core(wi, v, gam[w], sb[w], int(slots[w]))
            out = orc.decode_sg_core(wi, code, rG, sf, X[n - 1, j]).astype(np.float64)
            acc[j] += out
            e1 += ((out - truth[j]) ** 2).sum()
    den = (truth ** 2).sum()
    err1 = e1 / R / den
    errR = ((acc / R - truth) ** 2).sum() / den
    return err1, (errR - err1 / R) / (1.0 - 1.0 / R) / err1


def oracle_law(n):
    ctx = {}

    def slots(r, j):
        orc = ctx.setdefault(r, O.Oracle(n, seed=77, round=r))
        return [orc.draw_sg(j, w)[2] for w in range(n)]
    return slots


def ideal_law(n, seed=5):
    rng = np.random.default_rng(seed)
    return lambda r, j: rng.permutation(n)


def stride_law(n, seed=6):
    rng = np.random.default_rng(seed)
    m = max(1, int(n * 0.6180339887))
    while math.gcd(m, n) != 1:
        m += 1
    return lambda r, j: [(m * w + int(c)) % n for c in [rng.integers(0, n)] for w in range(n)]


@pytest.mark.parametrize("n,R,n_sg", [(8, 192, 12), (64, 64, 6)])
@pytest.mark.parametrize("wi", [0, 1, 2])
def test_multi_hop_bias_matches_an_ideal_shuffle_and_stays_small(n, R, n_sg, wi):
    e_law, b_law = ring_beta(n, wi, oracle_law(n), R, n_sg)
    e_ideal, b_ideal = ring_beta(n, wi, ideal_law(n), R, n_sg)
    assert 0.85 < e_law / e_ideal < 1.18, (e_law, e_ideal)
    assert b_law < BETA_BOUND and b_ideal < BETA_BOUND, (b_law, b_ideal)
    assert abs(b_law - b_ideal) < 0.008, (b_law, b_ideal)


@pytest.mark.parametrize("n,R,n_sg", [(8, 192, 12), (64, 64, 6)])
def test_a_fixed_stride_permutation_would_show(n, R, n_sg):
    """Negative control at 4 bits: slots of consecutive ring hops a fixed distance apart."""
    _, b_stride = ring_beta(n, 1, stride_law(n), R, n_sg)
    _, b_law = ring_beta(n, 1, oracle_law(n), R, n_sg)
    assert b_stride > BETA_BOUND and b_stride > 3.0 * max(b_law, 0.005), (b_stride, b_law)
