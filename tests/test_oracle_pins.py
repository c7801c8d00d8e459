"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each one is chosen so that a
plausible mistake in the oracle (a dropped term, a wrong sign or index, a
transposed operand, a biased rounding) makes it fail.
"""
import math
import os

import numpy as np
import pytest

from oracle import dq_oracle as O
from oracle import mini_oracle as M


def load_golden(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "paper_worked_examples.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, val, _ = [s.strip() for s in line.split("|", 2)]
            vals[name] = float(val)
    return vals


# ----------------------------------------------------------------- Philox (Salmon et al.)

def test_philox_known_answers(golden_dir):
    n = 0
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(x, 16) for x in line.split()]
            got = O.philox4x32_10(w[0:4], w[4:6])
            assert [int(x) for x in got] == w[6:10]
            assert M.philox(w[0:4], w[4:6]) == w[6:10]
            n += 1
    assert n == 3


# ----------------------------------------------------------------- level set (Section 3.3)

@pytest.mark.parametrize("wi,g", [(1, 1.3), (1, 2.0), (2, 1.02), (2, 1.05), (1, 1.0001)])
def test_levels_closed_form_properties(wi, g):
    rc, T, D = O.levels(wi, g)
    assert rc == 0
    R = O.RMAX[wi]
    assert T[0] == 0.0 and T[R] == 1.0
    assert np.all(np.diff(T.astype(np.float64)) > 0)
    # consecutive gaps grow by the factor 1+2eps^2:  f(r+2)-f(r+1) = g * (f(r+1)-f(r))
    ratio = D[1:].astype(np.float64) / D[:-1].astype(np.float64)
    assert np.allclose(ratio, g, rtol=2e-4 if wi == 2 else 1e-5)
    # f(eps, r) * (g^R - 1) + 1 = g^r
    pw = T.astype(np.float64) * (g ** R - 1.0) + 1.0
    assert np.allclose(pw, g ** np.arange(R + 1), rtol=1e-5)


def test_levels_limits():
    # eps -> 0: uniformly spaced levels r/R
    for wi in (1, 2):
        rc, T, _ = O.levels(wi, 1.0 + 1e-7)
        R = O.RMAX[wi]
        assert rc == 0 and np.allclose(T, np.arange(R + 1) / R, atol=1e-5)
    # b = 2: one magnitude bit -> {0, 1}, whatever eps is
    rc, T, D = O.levels(0, 1.7)
    assert rc == 0 and list(T) == [0.0, 1.0] and list(D) == [1.0]
    # larger eps -> more levels close to zero
    _, Ta, _ = O.levels(1, 1.1)
    _, Tb, _ = O.levels(1, 1.6)
    assert np.all(Tb[1:-1] < Ta[1:-1])
    # degenerate g: levels collapse -> rejected
    assert O.levels(2, 1.0)[0] != 0


# ----------------------------------------------------------------- stochastic quantization (Sections 2.1, 2.3, 3.2)

def all_uniforms(orc):
    """Every value the entry uniform can take, as an (n, 256) array indexed [slot, byte]."""
    n = orc.n_workers
    return np.array([[orc.entry_uniform(s, b) for b in range(256)] for s in range(n)], np.float32)


def sq_moments(T, D, x, us):
    """Mean and variance of the de-quantized value over the given equally likely uniforms."""
    vals = np.array([T[O.sq_index(T, D, x, u)] for u in us], np.float64)
    return vals.mean(), vals.var()


def test_worked_example_nonuniform_levels(golden_dir):
    gold = load_golden(golden_dir)
    us = all_uniforms(O.Oracle(1)).ravel()
    X = [-1.0, 0.5, 1.0]

    def total_mse(T):
        T = np.array(T, np.float32)
        D = np.diff(T).astype(np.float32)
        tot = 0.0
        for x in X:  # sign handled separately: quantize |x| / max|X|
            vals = np.array([T[O.sq_index(T, D, abs(x), u)] for u in us], np.float64)
            tot += np.mean((np.sign(x) * vals - x) ** 2)
        return tot

    assert total_mse([0.0, 1.0]) == pytest.approx(gold["nonuniform_mse_uniform_levels"], abs=1e-12)
    assert total_mse([0.0, 0.5, 1.0]) == pytest.approx(gold["nonuniform_mse_fitted_levels"], abs=1e-12)


def test_worked_example_worst_case_variance(golden_dir):
    gold = load_golden(golden_dir)
    us = all_uniforms(O.Oracle(1)).ravel()
    xs = np.arange(0, 65) / 64.0
    T1, D1 = np.array([0, 1], np.float32), np.array([1], np.float32)
    var1 = [sq_moments(T1, D1, x, us)[1] for x in xs]
    assert max(var1) == pytest.approx(gold["onebit_worst_variance"], abs=1e-12)
    assert xs[int(np.argmax(var1))] == 0.5
    T2, D2 = np.array([0, 0.5, 1], np.float32), np.array([0.5, 0.5], np.float32)
    var2 = [sq_moments(T2, D2, x, us)[1] for x in xs]
    assert max(var2) == pytest.approx(gold["twobit_worst_variance"], abs=1e-12)
    assert xs[int(np.argmax(var2))] in (0.25, 0.75)
    # each added bit (a level between every two) cuts the worst case by 4x
    assert max(var1) / max(var2) == pytest.approx(4.0)


@pytest.mark.parametrize("wi", [0, 1, 2])
@pytest.mark.parametrize("n", [1, 4, 3])
def test_sq_unbiased_by_enumeration(wi, n):
    """E[xhat'] = x' (Section 3.3): enumerate every (slot, byte) outcome.  The 8-bit
    gamma makes P(up) a multiple of 1/(256 n) that brackets p, so the bias is at most
    D[r]/(512 n) in exact arithmetic (plus fp32 rounding)."""
    orc = O.Oracle(n)
    T, D = orc.T(wi), orc.D(wi)
    us = all_uniforms(orc).ravel()
    rng = np.random.default_rng(5)
    xs = list(rng.uniform(0, 1, 12).astype(np.float32)) + [0.0, 1.0, float(T[1]), float(T[-2])]
    for x in xs:
        x = float(np.float32(x))
        mean, _ = sq_moments(T, D, x, us)
        r_lo = int(np.searchsorted(T, x, side="right") - 1)
        gap = float(D[min(r_lo, len(D) - 1)])
        assert abs(mean - x) <= gap / (512.0 * n) + 4e-7, (wi, n, x, mean)
        # the two candidates are the neighbours of x in Q (Section 2.1)
        idx = {O.sq_index(T, D, x, u) for u in us[:: max(1, len(us) // 64)]}
        assert idx <= {r_lo, min(r_lo + 1, len(T) - 1)}
    # levels themselves are reproduced exactly
    for r in range(len(T)):
        assert {O.sq_index(T, D, float(T[r]), float(u)) for u in us[::17]} == {r}


# ----------------------------------------------------------------- correlated rounding (Sections 2.4, 3.3)

@pytest.mark.parametrize("n", [2, 3, 4, 7, 8, 64, 100, 1000, 8192])
def test_exactly_one_uniform_per_interval(n):
    """For every super-group the slots of the n workers are a permutation of 0..n-1 and
    u_i lies in [pi_i/n, (pi_i+1)/n): exactly one worker per interval (Section 3.3)."""
    orc = O.Oracle(n, seed=1234, round=3)
    for sg in (0, 1, 77, 2 ** 33 + 5) if n <= 100 else (5,):
        slots = [orc.draw_sg(sg, r)[2] for r in range(n)]
        assert sorted(slots) == list(range(n))
        for s in slots[:8]:
            for byte in (0, 1, 127, 255):
                u = float(orc.entry_uniform(s, byte))
                assert 0.0 < u < 1.0 and math.floor(u * n) == s
    # the permutation is drawn, not fixed: it varies with the super-group and the round
    perms = {tuple(orc.draw_sg(sg, r)[2] for r in range(min(n, 8))) for sg in range(64)}
    assert len(perms) > 1
    other = O.Oracle(n, seed=1234, round=4)
    assert [orc.draw_sg(sg, 0)[2] for sg in range(64)] != [other.draw_sg(sg, 0)[2] for sg in range(64)]
    # and shared: it does not depend on which worker asks (same words for every rank)
    assert orc.draw_sg(9, 0)[2] != orc.draw_sg(9, 1)[2]


def _perm_words(count, seed):
    return np.random.default_rng(seed).integers(0, 1 << 32, (count, 4), dtype=np.uint64).astype(np.uint32)


@pytest.mark.parametrize("n", [2, 3, 4, 5, 8, 12, 16])
def test_permutation_is_a_bijection_for_any_words(n):
    """Whatever the four words are (also all-zero, all-one and single-bit words), the n workers
    get the n slots once each."""
    words = list(_perm_words(200, n)) + [np.zeros(4, np.uint32), np.full(4, 0xFFFFFFFF, np.uint32)]
    words += [np.array([1 << i, 1 << (31 - i), 1 << ((i + 16) % 32), 0], np.uint32) for i in range(32)]
    for w in words:
        assert sorted(O.perm_slot(w, n, r) for r in range(n)) == list(range(n))
    if n <= 4:  # every permutation of a small n is reachable
        assert len({tuple(O.perm_slot(w, n, r) for r in range(n)) for w in _perm_words(3000, 1)}) == math.factorial(n)


@pytest.mark.parametrize("n", [3, 8, 64, 100])
def test_permutation_marginals_and_pairs_look_uniform(n):
    """What a uniformly random permutation guarantees and an affine or fixed-stride map does not:
    every worker's slot is uniform on 0..n-1, the difference of two workers' slots is spread over
    all non-zero residues, and consecutive differences are not tied to each other."""
    N = 20000
    W = _perm_words(N, 100 + n)
    p = np.array([[O.perm_slot(w, n, r) for r in range(3)] for w in W])
    marg = np.bincount(p[:, 1], minlength=n)
    chi_m = ((marg - N / n) ** 2 / (N / n)).sum() / (n - 1)
    assert chi_m < 1.0 + 5.0 * math.sqrt(2.0 / (n - 1))          # chi-square per degree of freedom: 1 +- sqrt(2/dof)
    d = np.bincount((p[:, 1] - p[:, 0]) % n, minlength=n)
    assert d[0] == 0
    rel = d[1:] / (N / (n - 1))
    assert rel.min() > 0.7 and rel.max() < 1.3                    # a stride or a small multiplier would leave most residues empty
    if n > 3:
        same = np.mean((p[:, 2] - p[:, 1]) % n == (p[:, 1] - p[:, 0]) % n)
        assert abs(same - 1.0 / (n - 2)) < 0.35 / (n - 2) + 4.0 / math.sqrt(N)   # an affine map gives 1


def test_streams_are_private_or_shared_as_specified():
    orc = O.Oracle(4, seed=9)
    g0, s0, _ = orc.draw_sg(5, 0)
    g1, s1, _ = orc.draw_sg(5, 1)
    assert not np.array_equal(g0, g1) and not np.array_equal(s0, s1)  # gamma and scale bytes are per worker
    g0b, s0b, _ = orc.draw_sg(6, 0)
    assert not np.array_equal(g0, g0b) and not np.array_equal(s0, s0b)
    # bytes look uniform: mean 127.5 +- 5 sigma over 256*64 draws
    allg = np.concatenate([orc.draw_sg(sg, 2)[0] for sg in range(64)]).astype(np.float64)
    assert abs(allg.mean() - 127.5) < 5 * 73.9 / math.sqrt(allg.size)
    # no reuse between the gamma bytes of a group and the scale bytes of its super-group
    assert not np.array_equal(g0[:16], s0)


def two_worker_sg(value):
    v = np.full(256, value, np.float32)
    v[::16] = 1.0  # every group's maximum is 1, so normalisation is the identity
    return v


def test_worked_example_two_workers_cancel(golden_dir):
    """x1 = x2 = 1/2, one magnitude bit, shared permutation: the two roundings always go
    opposite ways, so the decoded sum is exactly 1 for every seed and super-group."""
    gold = load_golden(golden_dir)
    v = two_worker_sg(0.5)
    sums = []
    for seed in range(40):
        orc = O.Oracle(2, seed=seed)
        for sg in (0, 3):
            dec = []
            for rank in (0, 1):
                gamma, sb, slot = orc.draw_sg(sg, rank)
                code, rG, sf = orc.encode_sg_core(0, v, gamma, sb, slot)
                assert sf == 0x3F80 and np.all(rG == 255)
                dec.append(orc.decode_sg_core(0, code, rG, sf))
            sums.append(dec[0] + dec[1])
    sums = np.array(sums)
    half = np.ones(256, bool)
    half[::16] = False
    assert np.all(sums[:, ~half] == 2.0)
    assert np.all(sums[:, half] == 1.0)
    assert sums[:, half].var() == gold["correlated_pair_variance"]


def test_worked_example_independent_pair_variance(golden_dir):
    """Same inputs with independent uniforms (two single-worker contexts with different
    seeds): Var[x1hat + x2hat] = 1/2."""
    gold = load_golden(golden_dir)
    v = two_worker_sg(0.5)
    half = np.ones(256, bool)
    half[::16] = False
    sums = []
    for seed in range(60):
        a, b = O.Oracle(1, seed=2 * seed), O.Oracle(1, seed=2 * seed + 1)
        dec = []
        for orc in (a, b):
            gamma, sb, slot = orc.draw_sg(0, 0)
            code, rG, sf = orc.encode_sg_core(0, v, gamma, sb, slot)
            dec.append(orc.decode_sg_core(0, code, rG, sf))
        sums.append((dec[0] + dec[1])[half])
    sums = np.concatenate(sums).astype(np.float64)  # 60*240 samples in {0,1,2}
    assert sums.var() == pytest.approx(gold["independent_pair_variance"], rel=0.05)
    assert sums.mean() == pytest.approx(1.0, abs=0.02)


def test_correlated_pair_worst_case_variance(golden_dir):
    """Negative correlation, any x1, x2 in [0,1], one bit each: Var[x1hat+x2hat] <= 1/4.
    Enumerated exactly over the shared shift and both workers' bytes."""
    gold = load_golden(golden_dir)
    orc = O.Oracle(2)
    U = all_uniforms(orc).astype(np.float64)  # [slot, byte]
    worst = 0.0
    grid = np.arange(0, 17) / 16.0
    for x1 in grid:
        for x2 in grid:
            tot = []
            for shift in (0, 1):
                up1 = (U[(0 + shift) % 2] < x1).astype(np.float64)
                up2 = (U[(1 + shift) % 2] < x2).astype(np.float64)
                tot.append(up1[:, None] + up2[None, :])
            tot = np.stack(tot)
            worst = max(worst, tot.var())
            assert abs(tot.mean() - (x1 + x2)) <= 2.0 / 1024 + 1e-12
    assert worst <= gold["correlated_pair_worst_variance"] + 1e-12


# ----------------------------------------------------------------- hierarchical scales (Section 3.3)

def test_group_scale_unbiased_by_enumeration():
    """E[sf_G] = max|G|: enumerate the 256 scale bytes; the decoded group scale
    r_G*sf_SG/255 averages to the group maximum within (sf_SG/255)/512."""
    orc = O.Oracle(4, seed=3)
    rng = np.random.default_rng(11)
    v = (rng.standard_normal(256) * np.repeat(10.0 ** rng.uniform(-3, 0, 16), 16)).astype(np.float32)
    gamma, _, slot = orc.draw_sg(0, 0)
    r_sum = np.zeros(16)
    for byte in range(256):
        _, rG, sf = orc.encode_sg_core(1, v, gamma, np.full(16, byte, np.uint8), slot)
        r_sum += rG
    sf_f = float(np.array([sf << 16], np.uint32).view(np.float32)[0])
    m = np.abs(v).reshape(16, 16).max(axis=1).astype(np.float64)
    assert sf_f >= m.max() and sf_f <= m.max() * (1 + 2.0 ** -7)  # bf16, rounded up
    step = sf_f / 255.0
    assert np.all(np.abs(r_sum / 256.0 * step - m) <= step / 512.0 + 1e-6 * sf_f)
    # the rounded-up bf16 scale never lets r_G overflow and the largest group gets (nearly) 255
    assert r_sum.max() / 256.0 <= 255.0 and r_sum.max() / 256.0 >= 253.0


def test_bf16_round_up():
    for x, want in [(1.0, 0x3F80), (1.0000001, 0x3F81), (0.0, 0), (3.0e-3, None), (65280.0, 0x477F), (65281.0, 0x4780)]:
        h = O.bf16_ceil(x)
        if want is not None:
            assert h == want
        back = float(np.array([h << 16], np.uint32).view(np.float32)[0])
        assert back >= np.float32(x) and back <= np.float32(x) * (1 + 2.0 ** -7)


@pytest.mark.parametrize("wi", [0, 1, 2])
def test_full_path_unbiased_statistically(wi):
    """Compress -> decompress over many seeds: the sample mean converges to the input
    (unbiasedness survives the product of the two independent roundings, Section 3.3)."""
    rng = np.random.default_rng(17)
    v = (rng.standard_normal(256) * 1e-3).astype(np.float32)
    v[48:64] *= 0.01   # a quiet group
    v[100] *= 30.0     # an outlier
    N = 1500
    acc = np.zeros(256)
    acc2 = np.zeros(256)
    for seed in range(N):
        orc = O.Oracle(4, seed=seed)
        gamma, sb, slot = orc.draw_sg(seed % 7, seed % 4)
        code, rG, sf = orc.encode_sg_core(wi, v, gamma, sb, slot)
        d = orc.decode_sg_core(wi, code, rG, sf).astype(np.float64)
        acc += d
        acc2 += d * d
    mean = acc / N
    var = np.maximum(acc2 / N - mean ** 2, 0.0)
    # statistical tolerance + the enumerable bias of the 8-bit gamma (at most gap/(512 n)
    # of the group scale) + a floor for events rarer than 1/N
    m_g = np.repeat(np.abs(v).reshape(16, 16).max(axis=1), 16).astype(np.float64)
    tol = 4.5 * np.sqrt(var / N) + m_g * (1.0 / 2048.0) + 4.5 * m_g / N
    assert np.all(np.abs(mean - v) <= tol)
    assert abs(np.sum(mean - v)) <= 4.5 * np.sqrt(np.sum(m_g ** 2) / N)


@pytest.mark.parametrize("wi", [0, 1, 2])
def test_deterministic_error_bound(wi):
    """Given the realised scales: the de-quantized normalised value is a neighbour level of
    x' (error below the local gap) and |sf_G - max|G|| < sf_SG/255."""
    orc = O.Oracle(8, seed=2)
    T, D = orc.T(wi).astype(np.float64), orc.D(wi).astype(np.float64)
    R = O.RMAX[wi]
    rng = np.random.default_rng(23)
    for sg in range(6):
        v = (rng.standard_normal(256) * np.repeat(10.0 ** rng.uniform(-4, -1, 16), 16)).astype(np.float32)
        gamma, sb, slot = orc.draw_sg(sg, sg % 8)
        code, rG, sf = orc.encode_sg_core(wi, v, gamma, sb, slot)
        sf_f = float(np.array([sf << 16], np.uint32).view(np.float32)[0])
        m = np.abs(v).reshape(16, 16).max(axis=1).astype(np.float64)
        sfg = rG.astype(np.float64) * sf_f / 255.0
        assert np.all(np.abs(sfg - m) < sf_f / 255.0 * (1 + 1e-6))
        sign = code >> (O.BITS[wi] - 1)
        r = code & R
        assert np.array_equal(sign, (v < 0).astype(np.uint8) | (np.signbit(v)).astype(np.uint8))
        for g in range(16):
            if rG[g] == 0:
                assert np.all(r[g * 16:(g + 1) * 16] == 0)
                continue
            x = np.abs(v[g * 16:(g + 1) * 16]).astype(np.float64) / m[g]
            rr = r[g * 16:(g + 1) * 16]
            lo = np.searchsorted(T, x * (1 - 1e-7), side="right") - 1
            assert np.all((rr >= lo) & (rr <= np.minimum(lo + 1, R) + (x * (1 + 1e-7) >= T[np.minimum(lo + 1, R)])))
            assert np.all(np.abs(T[rr] - x) <= D[np.minimum(lo, R - 1)] * (1 + 1e-6) + 1e-7)


# ----------------------------------------------------------------- special cases

def test_zero_and_tiny_super_groups():
    orc = O.Oracle(4)
    gamma, sb, slot = orc.draw_sg(0, 0)
    for wi in range(3):
        v = np.zeros(256, np.float32)
        v[3] = -0.0
        code, rG, sf = orc.encode_sg_core(wi, v, gamma, sb, slot)
        assert sf == 0 and not rG.any()
        assert code[3] == 1 << (O.BITS[wi] - 1) and not np.delete(code, 3).any()
        out = orc.decode_sg_core(wi, code, rG, sf)
        assert np.all(out == 0.0)
        # magnitudes below 2^-100 are flushed (their reciprocals would overflow)
        v = np.full(256, 2.0 ** -110, np.float32)
        code, rG, sf = orc.encode_sg_core(wi, v, gamma, sb, slot)
        assert sf == 0 and not rG.any() and not code.any()
        # one zero group inside a live super-group
        v = np.ones(256, np.float32)
        v[16:32] = 0.0
        code, rG, sf = orc.encode_sg_core(wi, v, gamma, sb, slot)
        assert rG[1] == 0 and not code[16:32].any() and np.all(rG[[0, 2, 15]] == 255)
        assert np.all(orc.decode_sg_core(wi, code, rG, sf)[16:32] == 0.0)


def test_denormal_group_in_live_super_group():
    orc = O.Oracle(2)
    gamma, sb, slot = orc.draw_sg(0, 0)
    v = np.full(256, 1e-3, np.float32)
    v[32:48] = 1e-42  # denormals: 1/m overflows, but r_G is 0 so the entries are never normalised
    for wi in range(3):
        code, rG, sf = orc.encode_sg_core(wi, v, gamma, sb, slot)
        assert rG[2] == 0 and not code[32:48].any()
        assert np.all(np.isfinite(orc.decode_sg_core(wi, code, rG, sf)))


def test_two_bit_width_is_ternary():
    orc = O.Oracle(4, seed=8)
    rng = np.random.default_rng(2)
    v = rng.standard_normal(256).astype(np.float32)
    gamma, sb, slot = orc.draw_sg(1, 2)
    code, rG, sf = orc.encode_sg_core(0, v, gamma, sb, slot)
    out = orc.decode_sg_core(0, code, rG, sf)
    sf_f = float(np.array([sf << 16], np.uint32).view(np.float32)[0])
    for g in range(16):
        sfg = np.float32(rG[g]) * (np.float32(sf_f) / np.float32(255.0))
        assert set(np.unique(out[g * 16:(g + 1) * 16])) <= {np.float32(0.0), sfg, -sfg}


def test_single_worker_is_plain_sq():
    """n = 1: the permutation is trivial and u = gamma = (byte + 1/2)/256."""
    orc = O.Oracle(1, seed=77)
    for sg in range(5):
        assert orc.draw_sg(sg, 0)[2] == 0
    for byte in (0, 1, 200, 255):
        assert orc.entry_uniform(0, byte) == (byte + 0.5) / 256.0


@pytest.mark.parametrize("wi", [1, 2])
def test_lattice_input_is_lossless(wi):
    """Entries that sit exactly on the lattice sf_G*T[r], with group maxima the codec can
    represent exactly, survive compress -> decompress unchanged."""
    orc = O.Oracle(4, seed=4)
    T = orc.T(wi)
    R = O.RMAX[wi]
    rng = np.random.default_rng(9)
    r = rng.integers(0, R + 1, 256)
    r[::16] = R  # each group holds its maximum
    sign = rng.integers(0, 2, 256)
    scale = np.float32(0.5)  # sf_SG = 0.5, every r_G = 255, sf_G = 255*(0.5/255) = 0.5 exactly
    assert np.float32(255.0) * (scale / np.float32(255.0)) == scale
    v = (np.where(sign == 1, -1.0, 1.0) * T[r].astype(np.float64) * float(scale)).astype(np.float32)
    gamma, sb, slot = orc.draw_sg(9, 1)
    code, rG, sf = orc.encode_sg_core(wi, v, gamma, sb, slot)
    assert np.all(rG == 255) and sf == 0x3F00
    out = orc.decode_sg_core(wi, code, rG, sf)
    nz = r > 0
    assert np.array_equal(out[nz], v[nz]) and np.all(out[~nz] == 0.0)
    assert np.array_equal(code & R, r)


# ----------------------------------------------------------------- bit accounting and wire format (Section 3.5)

def test_bit_accounting(golden_dir):
    gold = load_golden(golden_dir)
    assert 32 / 256 == gold["budget5_stats_bits"]
    assert 8 / 16 == gold["budget5_group_scale_bits"]
    assert 16 / 256 == gold["budget5_sg_scale_bits"]
    assert 5 - 32 / 256 - 8 / 16 - 16 / 256 == gold["budget5_code_bits"]
    # 6400 super-groups averaging 4.3125 code bits: 5900 at 4 bits, 500 at 8 bits
    ch = O.make_chunk(0, [0, 5900, 500])
    assert (4 * 5900 + 8 * 500) / 6400 == gold["budget5_code_bits"]
    bits_per_entry = O.Oracle.packed_bytes(ch) * 8 / (6400 * 256)
    assert bits_per_entry == gold["budget5_main_bits"]
    # sizes per width
    assert O.Oracle.packed_bytes(O.make_chunk(0, [8, 0, 0])) == 8 * (64 + 18)
    assert O.Oracle.packed_bytes(O.make_chunk(0, [0, 8, 0])) == 8 * (128 + 18)
    assert O.Oracle.packed_bytes(O.make_chunk(0, [0, 0, 8])) == 8 * (256 + 18)
    assert O.Oracle.packed_bytes(O.make_chunk(0, [1, 0, 0])) == 96  # 82 rounded up to 16


def test_wire_layout_matches_core_encoder():
    """compress() = encode_sg_core per super-group + the documented layout."""
    orc = O.Oracle(4, seed=21, round=2)
    n_sg = [2, 3, 1]
    ch = O.make_chunk(1000, n_sg)
    rng = np.random.default_rng(3)
    local = (rng.standard_normal(6 * 256) * 1e-2).astype(np.float32)
    packed = orc.compress(ch, 3, local)
    off = [0, 2 * 64, 2 * 64 + 3 * 128]
    gs_off = off[2] + 256
    sg_off = gs_off + 16 * 6
    assert packed.size == ((sg_off + 12 + 15) // 16) * 16
    j = 0
    for wi in range(3):
        b = O.BITS[wi]
        for pos in range(n_sg[wi]):
            gamma, sb, slot = orc.draw_sg(1000 + j, 3)
            code, rG, sf = orc.encode_sg_core(wi, local[j * 256:(j + 1) * 256], gamma, sb, slot)
            blk = packed[off[wi] + pos * 32 * b: off[wi] + (pos + 1) * 32 * b]
            bits = np.unpackbits(blk, bitorder="little").reshape(256, b)
            got = (bits * (1 << np.arange(b))).sum(axis=1)
            assert np.array_equal(got, code)
            assert np.array_equal(packed[gs_off + 16 * j: gs_off + 16 * (j + 1)], rG)
            assert int(packed[sg_off + 2 * j]) | (int(packed[sg_off + 2 * j + 1]) << 8) == sf
            j += 1


def test_bf16_local_equals_widened_fp32_local():
    orc = O.Oracle(4, seed=5)
    ch = O.make_chunk(0, [1, 2, 1])
    rng = np.random.default_rng(8)
    h = (rng.standard_normal(4 * 256).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    wide = (h.astype(np.uint32) << 16).view(np.float32)
    p16 = orc.compress(ch, 1, h)
    p32 = orc.compress(ch, 1, wide)
    assert np.array_equal(p16, p32)
    assert np.array_equal(orc.dar_hop(ch, 2, p16, h), orc.dar_hop(ch, 2, p32, wide))
    assert np.array_equal(orc.decompress(ch, p16, h), orc.decompress(ch, p32, wide))


def test_mean_is_subtracted_in_fp32_where_the_entry_enters():
    """Section 3.1: a call with means equals the same call on entries from which the mean was
    taken off beforehand in fp32 (never rounded back to bf16), for every kernel and width."""
    orc = O.Oracle(4, seed=9)
    ch = O.make_chunk(3, [1, 2, 1, 1])
    rng = np.random.default_rng(12)
    h = ((rng.standard_normal(5 * 256) * 0.01).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    wide = (h.astype(np.uint32) << 16).view(np.float32)
    mu = (rng.standard_normal(5) * 1e-3).astype(np.float32)
    pre = wide - np.repeat(mu, 256)                      # one fp32 subtraction per entry
    assert not np.array_equal(pre, wide)
    p = orc.compress(ch, 1, h, mu)
    assert np.array_equal(p, orc.compress(ch, 1, pre))
    assert np.array_equal(p, orc.compress(ch, 1, wide, mu))
    assert not np.array_equal(p, orc.compress(ch, 1, h))
    assert np.array_equal(orc.dar_hop(ch, 2, p, h, mu), orc.dar_hop(ch, 2, p, pre))
    assert np.array_equal(orc.decompress(ch, p, h, mu), orc.decompress(ch, p, pre))
    assert np.array_equal(orc.decompress(ch, p, None, mu), orc.decompress(ch, p))   # no local: nothing to subtract


def test_constant_super_group_minus_its_mean_is_zero():
    """A wrong sign (x + mu) or a mean taken from the wrong super-group would leave 2c or c."""
    orc = O.Oracle(2, seed=1)
    ch = O.make_chunk(0, [1, 1, 1])
    c = np.array([0.375, -2.5, 7.0], np.float32)
    x = np.repeat(c, 256)
    p = orc.compress(ch, 0, x, c)
    assert not np.any(orc.decompress(ch, p))
    got = orc.decompress(ch, p, x, c[::-1].copy())       # decode 0 + (x - other mean): exact differences
    assert np.array_equal(got, x - np.repeat(c[::-1], 256))


# ----------------------------------------------------------------- independent re-implementation

@pytest.mark.parametrize("b,wi", [(2, 0), (4, 1), (8, 2)])
@pytest.mark.parametrize("n", [1, 3, 4])
def test_c_oracle_matches_pure_python_oracle(b, wi, n):
    g = {2: 2.0, 4: 1.3, 8: 1.02}[b]
    seed, rnd = 0x1234567890ABCDEF, 7
    orc = O.Oracle(n, seed=seed, round=rnd, g4=1.3, g8=1.02)
    rng = np.random.default_rng(100 + b + n)
    for sg in (0, 2 ** 32 + 3):
        rank = (sg + 1) % n
        v = (rng.standard_normal(256) * np.repeat(10.0 ** rng.uniform(-5, 0, 16), 16)).astype(np.float32)
        v[17] = 0.0
        gamma, sb, slot = orc.draw_sg(sg, rank)
        mg, ms, mslot = M.draws(seed, rnd, n, sg, rank)
        assert list(gamma) == mg and list(sb) == ms and slot == mslot
        code, rG, sf = orc.encode_sg_core(wi, v, gamma, sb, slot)
        mcode, mrG, msf = M.encode_sg(b, g, n, seed, rnd, sg, rank, v)
        assert list(code) == mcode and list(rG) == mrG and sf == msf
        local = (rng.standard_normal(256) * 1e-2).astype(np.float32)
        assert np.array_equal(orc.decode_sg_core(wi, code, rG, sf), M.decode_sg(b, g, mcode, mrG, msf))
        assert np.array_equal(orc.decode_sg_core(wi, code, rG, sf, local), M.decode_sg(b, g, mcode, mrG, msf, local))


def test_mini_oracle_rounding_helper():
    # the exact-rational fused multiply-add against cases with known answers
    f = np.float32
    assert M.fma32(f(1 + 2 ** -12), f(1 + 2 ** -12), f(-1.0)) == f(2 ** -11 + 2 ** -24)  # exact, no intermediate rounding
    assert M.round_to_f32(M.Fraction(1) + M.Fraction(1, 2 ** 24)) == f(1.0)              # tie -> even
    assert M.round_to_f32(M.Fraction(1) + M.Fraction(3, 2 ** 24)) == f(1 + 2 ** -22)     # tie -> even (up)
    assert M.round_to_f32(M.Fraction(1, 2 ** 149)) == f(2.0 ** -149)                      # smallest subnormal
    assert M.round_to_f32(M.Fraction(1, 2 ** 150)) == f(0.0)                              # tie -> even (zero)


def test_groups_of_a_worker_are_spread_over_the_intervals():
    """pi advances by one per group: with n = 16, identical groups, identical gamma bytes and
    x' = 1/2, exactly the 8 groups whose slot is below n/2 round up."""
    orc = O.Oracle(16, seed=12)
    v = two_worker_sg(0.5)
    for rank in (0, 5):
        _, sb, slot = orc.draw_sg(2, rank)
        code, rG, _ = orc.encode_sg_core(0, v, np.full(256, 128, np.uint8), sb, slot)
        ups = code.reshape(16, 16)[:, 1]  # entry 1 of every group (entry 0 is the group maximum)
        want = [1 if (slot + g) % 16 < 8 else 0 for g in range(16)]
        assert list(ups) == want and sum(want) == 8


# ----------------------------------------------------------------- the fused hop (Section 3.4 "Fused kernels"; Section 4, kernel 3)

def _hop_case(dtype, n_sg, seed):
    """A chunk, an incoming message from worker 1, a local slice of `dtype` and per-SG means."""
    rng = np.random.default_rng(seed)
    total = sum(n_sg)
    ch = O.make_chunk(2 ** 32 + 7, n_sg)
    first = (rng.standard_normal(total * 256) * np.repeat(10.0 ** rng.uniform(-4, -1, total * 16), 16)).astype(np.float32)
    local = (rng.standard_normal(total * 256) * np.repeat(10.0 ** rng.uniform(-4, -1, total * 16), 16)).astype(np.float32)
    local[40:56] = 0.0  # a silent group: the decoded value alone survives
    if dtype == np.uint16:
        local = (local.view(np.uint32) >> 16).astype(np.uint16)
    mu = (rng.standard_normal(total) * 1e-4).astype(np.float32)
    return ch, first, local, mu


def _widen(a):
    return a if a.dtype == np.float32 else (a.astype(np.uint32) << 16).view(np.float32)


HOP_SHAPES = [[3, 0, 0], [0, 3, 0], [0, 0, 3], [2, 3, 1], [1, 2, 1, 2]]


@pytest.mark.parametrize("n_sg", HOP_SHAPES)
@pytest.mark.parametrize("dtype", [np.float32, np.uint16])
@pytest.mark.parametrize("with_mu", [False, True])
def test_dar_hop_is_decompress_accumulate_then_compress(n_sg, dtype, with_mu):
    """The fused kernel is by definition decompress -> accumulate -> recompress with nothing
    materialised in between: its bytes equal compress(rank, decompress(packed, local, mu)).
    The fp32 array in the middle holds exactly the values the hop keeps in registers."""
    n = 8
    orc = O.Oracle(n, seed=31, round=5)
    ch, first, local, mu = _hop_case(dtype, n_sg, 40 + len(n_sg) + sum(n_sg))
    m = mu if with_mu else None
    packed = orc.compress(ch, 1, first)
    for rank in (2, 7):
        mid = orc.decompress(ch, packed, local, m)
        want = orc.compress(ch, rank, mid)           # no means: mid is a sum, its means are already off
        got = orc.dar_hop(ch, rank, packed, local, m)
        assert np.array_equal(got, want)
        packed = got                                  # the next hop re-encodes what this one sent


@pytest.mark.parametrize("n_sg", HOP_SHAPES[:4])
@pytest.mark.parametrize("dtype", [np.float32, np.uint16])
@pytest.mark.parametrize("with_mu", [False, True])
def test_dar_hop_composed_by_hand_from_the_core_functions(n_sg, dtype, with_mu):
    """The same bytes from the pieces: unpack the documented layout, decode_sg_core with the
    mean-subtracted local super-group, the random numbers of THIS worker and of the
    super-group's global index (draw_sg(first_sg + j, rank)), encode_sg_core, pack.  Drawing
    with the sender's rank, with a chunk-relative index or skipping the mean gives other bytes."""
    n = 8
    sender, rank = 1, 5
    orc = O.Oracle(n, seed=77, round=2)
    ch, first, local, mu = _hop_case(dtype, n_sg, 60 + sum(n_sg))
    packed = orc.compress(ch, sender, first)
    got = orc.dar_hop(ch, rank, packed, local, mu if with_mu else None)
    total = sum(n_sg)
    code_off = np.cumsum([0] + [n_sg[w] * 32 * O.BITS[w] for w in range(3)])
    gs_off = int(code_off[3])
    sf_off = gs_off + 16 * total

    def compose(draw_rank, index_base, use_mu):
        out = np.zeros(got.size, np.uint8)
        wide = _widen(local)
        j = 0
        for wi in range(3):
            b = O.BITS[wi]
            for pos in range(n_sg[wi]):
                blk = packed[code_off[wi] + pos * 32 * b: code_off[wi] + (pos + 1) * 32 * b]
                bits = np.unpackbits(blk, bitorder="little").reshape(256, b)
                code_in = (bits * (1 << np.arange(b))).sum(axis=1).astype(np.uint8)
                rG_in = packed[gs_off + 16 * j: gs_off + 16 * (j + 1)]
                sf_in = int(packed[sf_off + 2 * j]) | (int(packed[sf_off + 2 * j + 1]) << 8)
                loc = wide[j * 256:(j + 1) * 256]
                if use_mu:
                    loc = loc - mu[j]                                   # one fp32 subtraction per entry
                v = orc.decode_sg_core(wi, code_in, rG_in, sf_in, loc)  # decode + accumulate
                gamma, sb, slot = orc.draw_sg(index_base + j, draw_rank)
                code, rG, sf = orc.encode_sg_core(wi, v, gamma, sb, slot)
                cb = np.unpackbits(code.reshape(256, 1), axis=1, bitorder="little")[:, :b]
                out[code_off[wi] + pos * 32 * b: code_off[wi] + (pos + 1) * 32 * b] = np.packbits(cb.ravel(), bitorder="little")
                out[gs_off + 16 * j: gs_off + 16 * (j + 1)] = rG
                out[sf_off + 2 * j], out[sf_off + 2 * j + 1] = sf & 0xFF, sf >> 8
                j += 1
        return out

    assert np.array_equal(got, compose(rank, ch.first_sg, with_mu))
    # negative controls: each plausible mistake changes the bytes
    assert not np.array_equal(got, compose(sender, ch.first_sg, with_mu))     # the sender's rank
    assert not np.array_equal(got, compose(rank, 0, with_mu))                 # chunk-relative index
    assert not np.array_equal(got, compose(rank, ch.first_sg, not with_mu))   # mean skipped / applied


def test_dar_hop_with_zero_message_is_compress_and_in_place():
    """Decoding an all-zero message adds nothing: the hop then equals the leaf's compress of the
    local slice with the hop's rank; and writing over the incoming buffer changes nothing."""
    orc = O.Oracle(4, seed=3)
    ch, _, local, mu = _hop_case(np.uint16, [1, 2, 1, 1], 9)
    zero = orc.compress(ch, 0, np.zeros(5 * 256, np.float32))
    assert not zero.any()
    assert np.array_equal(orc.dar_hop(ch, 3, zero, local, mu), orc.compress(ch, 3, local, mu))
    packed = orc.compress(ch, 1, _widen(local)[::-1].copy())
    want = orc.dar_hop(ch, 2, packed, local, mu)
    buf = packed.copy()
    O.lib().dqo_dar_hop(orc.h, O.C.byref(ch), 2, O._p(buf), O._p(local), O.BF16, O._p(mu), O._p(buf))
    assert np.array_equal(buf, want)
