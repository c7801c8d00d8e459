"""Pins of the pre/post-stage oracle (oracle/pp_oracle.c) against what the paper and the
mathematics fix: closed forms, the printed threshold ratio, Appendix A's logarithmic rule,
brute force over every threshold that matters, a second implementation (prep.allocate),
library special cases (stable argsort, torch's bf16 cast), round trips."""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import pp_oracle as P
from paper_2602_08923_amd import prep

f32 = np.float32


def bf16_bits(a):
    """float32 array of values exactly representable in bf16 -> uint16 patterns"""
    b = np.asarray(a, np.float32).view(np.uint32)
    assert np.all(b & 0xFFFF == 0)
    return (b >> 16).astype(np.uint16)


# ---------------------------------------------------------------- statistics (Section 3.1)
def test_stats_closed_forms():
    c = 0.375
    ramp = np.arange(256, dtype=np.float64) * 2.0 ** -10
    x = np.concatenate([np.full(256, c), np.tile([0.5, -0.5], 128), ramp, np.zeros(256)]).astype(f32)
    mu, F = P.sg_stats(x)
    assert mu[0] == c and F[0] == 256 * c * c                       # constant
    assert mu[1] == 0.0 and F[1] == 256 * 0.25                      # alternating signs
    assert mu[2] == 127.5 * 2.0 ** -10                              # sum k = n(n-1)/2
    assert F[2] == 5559680 * 2.0 ** -20                             # sum k^2 = (n-1)n(2n-1)/6
    assert mu[3] == 0.0 and F[3] == 0.0
    mu_b, F_b = P.sg_stats(bf16_bits(x[:512]))                      # the same values as bf16 patterns
    assert np.array_equal(mu_b, mu[:2]) and np.array_equal(F_b, F[:2])


def test_stats_single_entry_and_sign():
    x = np.zeros(512, f32)
    x[7] = -3.0
    x[256 + 255] = 2.0
    mu, F = P.sg_stats(x)
    assert mu[0] == -3.0 / 256 and F[0] == 9.0        # a dropped sign or a squared mean would show
    assert mu[1] == 2.0 / 256 and F[1] == 4.0         # the last entry of a super-group belongs to it


def test_bf16_round_to_nearest_even():
    assert P.bf16_rne(1.0) == 0x3F80
    assert P.bf16_rne(1.0 + 2.0 ** -8) == 0x3F80          # tie -> even
    assert P.bf16_rne(1.0 + 3 * 2.0 ** -8) == 0x3F82      # tie -> even (up)
    assert P.bf16_rne(1.0 + 2.0 ** -8 + 2.0 ** -20) == 0x3F81
    assert P.bf16_rne(-0.75) == 0xBF40
    v = np.random.default_rng(1).standard_normal(4096).astype(f32) * f32(1e-3)
    want = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([P.bf16_rne(t) for t in v], np.uint16)
    assert np.array_equal(got, want)                      # library cast, same rounding mode


def test_combine_definition():
    # exactly representable statistics: mu_j = (1/n) sum mu_ij, F_j = sum F_ij (Section 3.1)
    mu_all = np.array([[0.5, -1.0, 0.0], [0.25, 1.0, 0.0], [0.75, 3.0, 0.0], [0.5, 1.0, 0.0]], f32)
    F_all = np.array([[1.0, 2.0, 0.0], [3.0, 0.5, 0.0], [4.0, 0.25, 0.0], [8.0, 0.125, 0.0]], f32)
    mu, F = P.stats_combine(mu_all, F_all)
    assert np.array_equal(mu, np.array([0.5, 1.0, 0.0], f32))
    assert np.array_equal(F, np.array([16.0, 2.875, 0.0], f32))


def test_combine_rounds_contributions_to_bf16():
    # each worker sends two BF16 numbers per super-group (Section 3.5)
    mu_all = np.array([[1.0 + 2.0 ** -8], [1.0 + 3 * 2.0 ** -8]], f32)     # -> 1.0 and 1.015625
    F_all = np.array([[257.0], [3.0]], f32)                                  # 257 -> 256 (tie to even)
    mu, F = P.stats_combine(mu_all, F_all)
    assert mu[0] == f32(2.015625) / f32(2.0) and F[0] == f32(259.0)


# ---------------------------------------------------------------- thresholds (Section 3.2)
def test_threshold_ratio_from_per_bit_benefits():
    # per-bit benefit of lowering T_{a,b}: T (4^(b-a) - 1) / (4^b (b-a)); equal benefits tie the thresholds
    def benefit(a, b):
        return Fraction(4 ** (b - a) - 1, 4 ** b * (b - a))
    assert benefit(2, 4) == Fraction(15, 512) and benefit(4, 8) == Fraction(255, 4 ** 9)
    ratio = benefit(4, 8) / benefit(2, 4)                 # T_{2,4} / T_{4,8}
    assert ratio == Fraction(17, 512)
    theta = f32(3.0)
    t24 = f32(3.0 * 17.0 / 512.0)                         # exact: 51/512
    assert P.width(theta, theta) == 8
    assert P.width(np.nextafter(theta, f32(0)), theta) == 4
    assert P.width(t24, theta) == 4
    assert P.width(np.nextafter(t24, f32(0)), theta) == 2
    assert P.width(0.0, theta) == 2
    assert P.width(1e30, np.inf) == 2                     # infinite threshold: everything at 2 bits


def test_widths_follow_appendix_a_rule():
    # q = 2^clamp([1,3], floor(log2(K log2 F + u))), K = 4 / log2(512/17); T_{4,8} = 2^((8-u)/K)
    K = 4.0 / math.log2(512.0 / 17.0)
    rng = np.random.default_rng(5)
    F = np.exp2(rng.uniform(-40, 10, 4000)).astype(f32)
    seen = set()
    for u in (5.0, 14.5, 23.25, 30.0):
        z = K * np.log2(F.astype(np.float64)) + u
        safe = (np.abs(z - 4) > 1e-4) & (np.abs(z - 8) > 1e-4) & (z > 1)   # away from the boundaries
        zz = np.where(z > 1, z, 2.0)
        q = 2 ** np.clip(np.floor(np.log2(zz)), 1, 3)
        q = np.where(z < 2, 2, q)                     # z < 2 clamps to 2 bits as well
        theta = f32(2.0 ** ((8.0 - u) / K))
        got = np.array([P.width(f, theta) for f in F])
        assert np.array_equal(got[safe], q[safe].astype(int))
        seen |= set(got[safe].tolist())
        assert len(set(got[safe].tolist())) >= 2
    assert seen == {2, 4, 8}


# ---------------------------------------------------------------- allocation (Appendix A)
def np_cost(F, theta):
    theta = f32(theta)
    t24 = f32(theta * f32(17.0 / 512.0))
    return 2 * F.size + 2 * int(np.sum(F >= t24)) + 4 * int(np.sum(F >= theta))


def neighbours(v, k=3):
    out = [f32(v)]
    lo = hi = f32(v)
    for _ in range(k):
        lo = np.nextafter(lo, f32(-np.inf))
        hi = np.nextafter(hi, f32(np.inf))
        out += [lo, hi]
    return [t for t in out if t > 0]


@pytest.mark.parametrize("seed", range(12))
def test_allocate_brute_force(seed):
    """The cost is a step function of the threshold that only drops just above some F_j or
    just above some F_j * 512/17: the smallest fitting threshold is one of those points."""
    rng = np.random.default_rng(seed)
    J = int(rng.integers(3, 40))
    F = np.exp(rng.normal(-6, 3, J)).astype(f32)
    if seed % 3 == 0:
        F[rng.integers(0, J, 3)] = 0                       # empty super-groups
    if seed % 4 == 1:
        F[: J // 2] = F[0]                                 # ties
    budget = int(rng.uniform(2.0, 8.3) * J)
    cands = [f32(np.inf), np.nextafter(f32(0), f32(1))]
    for f in F[F > 0]:
        cands += neighbours(f) + neighbours(f32(f) * f32(512.0 / 17.0), 6)
    cands = sorted(set(float(c) for c in cands))
    fits = [c for c in cands if np_cost(F, c) <= budget]
    w, tbits = P.allocate(F, budget)
    theta = np.array([tbits], np.uint32).view(f32)[0]
    assert float(theta) == min(fits)
    assert int(w.astype(int).sum()) == np_cost(F, theta) <= budget
    # one representable step down must break the budget (or there is no step down)
    if tbits > 1:
        below = np.array([tbits - 1], np.uint32).view(f32)[0]
        assert np_cost(F, below) > budget
    assert np.array_equal(w, np.array([P.width(f, theta) for f in F], np.uint8))


def test_allocate_budget_edges():
    F = np.array([1.0, 2.0, 4.0, 0.0], f32)
    with pytest.raises(ValueError):
        P.allocate(F, 7)                                   # below 2 bits each
    up = lambda v: np.nextafter(f32(v), f32(np.inf))
    bits = lambda v: int(np.array([v], f32).view(np.uint32)[0])
    w, t = P.allocate(F, 8)
    # all at 2 bits needs T_{2,4} = theta * 17/512 above the largest norm: the smallest such theta
    th = f32(4.0 * 512.0 / 17.0)
    while f32(th * f32(17.0 / 512.0)) > f32(4.0):
        th = np.nextafter(th, f32(0))
    assert list(w) == [2, 2, 2, 2] and t == bits(up(th))
    # the thresholds are tied: 8 bits for F = 4 alone would put T_{2,4} below 1 and 2 (cost 18)
    w, t = P.allocate(F, 14)
    assert list(w) == [4, 4, 4, 2] and t == bits(up(4.0))
    w, t = P.allocate(F, 18)
    assert list(w) == [4, 4, 8, 2] and t == bits(up(2.0))
    w, t = P.allocate(F, 32)
    assert list(w) == [8, 8, 8, 4] and t == 1             # everything fits: smallest positive threshold,
                                                          # whose T_{2,4} underflows to 0 and admits F = 0


def test_allocate_cost_monotone():
    rng = np.random.default_rng(9)
    F = np.exp(rng.normal(-6, 3, 500)).astype(f32)
    th = np.sort(np.exp(rng.normal(-3, 6, 200)).astype(f32))
    c = [P.cost(F, t) for t in th]
    assert all(a >= b for a, b in zip(c, c[1:]))
    assert [P.cost(F, t) for t in th[:20]] == [np_cost(F, t) for t in th[:20]]


@pytest.mark.parametrize("budget_bits", [3.0, 4.0, 5.0, 6.5])
def test_allocate_agrees_with_log_bisection(budget_bits):
    """Second implementation: the float64 bisection on Appendix A's offset u (prep.allocate)
    reaches the same allocation on data without ties at the thresholds."""
    rng = np.random.default_rng(int(budget_bits * 10))
    J = 4096
    F = np.exp(rng.normal(-14, 2.5, J)).astype(f32)
    want = prep.allocate(torch.from_numpy(F.astype(np.float64)), budget_bits).numpy()
    w, _ = P.allocate(F, int(math.floor(prep.code_bits(budget_bits) * J)))
    assert np.array_equal(w.astype(np.int64), want)


# ---------------------------------------------------------------- W = {2,4,8,16}
def np_cost16(F, theta):
    theta = f32(theta)
    t24 = f32(theta * f32(17.0 / 512.0))
    t816 = f32(theta * f32(131072.0 / 257.0))
    return 2 * F.size + 2 * int(np.sum(F >= t24)) + 4 * int(np.sum(F >= theta)) + 8 * int(np.sum(F >= t816))


def test_sixteen_bit_threshold_ratio():
    def benefit(a, b):
        return Fraction(4 ** (b - a) - 1, 4 ** b * (b - a))
    assert benefit(4, 8) / benefit(8, 16) == Fraction(2 ** 17, 257)      # T_{8,16} / T_{4,8} (Section 3.2)
    theta = f32(2.0 ** -20)
    t816 = f32(theta * f32(131072.0 / 257.0))
    assert P.width(t816, theta, 16) == 16 and P.width(t816, theta, 8) == 8
    assert P.width(np.nextafter(t816, f32(0)), theta, 16) == 8
    assert P.width(theta, theta, 16) == 8 and P.width(0.0, theta, 16) == 2
    assert P.width(1e30, np.inf, 16) == 2


@pytest.mark.parametrize("seed", range(8))
def test_allocate_with_sixteen_bits_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    J = int(rng.integers(3, 40))
    F = np.exp(rng.normal(-6, 3, J)).astype(f32)
    if seed % 3 == 0:
        F[rng.integers(0, J, 2)] = 0
    budget = int(rng.uniform(2.0, 14.0) * J)
    cands = [f32(np.inf), np.nextafter(f32(0), f32(1))]
    for f in F[F > 0]:
        cands += neighbours(f) + neighbours(f32(f) * f32(512.0 / 17.0), 6) + neighbours(f32(f) * f32(257.0 / 131072.0), 6)
    cands = sorted(set(float(c) for c in cands))
    fits = [c for c in cands if np_cost16(F, c) <= budget]
    w, tbits = P.allocate(F, budget, max_width=16)
    theta = np.array([tbits], np.uint32).view(f32)[0]
    assert float(theta) == min(fits)
    assert int(w.astype(int).sum()) == np_cost16(F, theta) <= budget
    if tbits > 1:
        assert np_cost16(F, np.array([tbits - 1], np.uint32).view(f32)[0]) > budget
    assert set(w.tolist()) <= {2, 4, 8, 16}
    order = np.argsort(F, kind="stable")
    assert np.all(np.diff(w[order].astype(int)) >= 0)


def test_sixteen_bits_go_to_the_largest_norms():
    rng = np.random.default_rng(77)
    F = np.exp(rng.normal(-10, 4, 4096)).astype(f32)
    w16, _ = P.allocate(F, int(7.8125 * 4096), max_width=16)
    w8, _ = P.allocate(F, int(7.8125 * 4096), max_width=8)
    assert (w16 == 16).sum() > 0 and F[w16 == 16].min() >= F[w16 != 16].max()
    assert set(w8.tolist()) <= {2, 4, 8}
    # the same budget with a 16-bit class moves bits from the middle to the top
    assert (w16 == 8).sum() < (w8 == 8).sum()


# ---------------------------------------------------------------- reorder / restore
def test_positions_are_the_stable_sort():
    rng = np.random.default_rng(3)
    w = rng.choice(np.array([2, 4, 8, 16], np.uint8), 1000, p=[0.5, 0.3, 0.15, 0.05])
    pos, counts = P.positions(w)
    perm = np.argsort(w, kind="stable")                    # reordered[k] = original[perm[k]]
    inv = np.empty_like(perm)
    inv[perm] = np.arange(perm.size)
    assert np.array_equal(pos.astype(np.int64), inv)
    assert counts == [int((w == b).sum()) for b in (2, 4, 8, 16)]
    assert sorted(pos.tolist()) == list(range(1000))
    ws = w[perm]
    assert np.all(np.diff(ws.astype(int)) >= 0)            # increasing width order (Section 3.5)


def test_positions_degenerate():
    pos, counts = P.positions(np.full(5, 4, np.uint8))
    assert pos.tolist() == [0, 1, 2, 3, 4] and counts == [0, 5, 0, 0]
    pos, counts = P.positions(np.zeros(0, np.uint8))
    assert pos.size == 0 and counts == [0, 0, 0, 0]


def test_reorder_moves_whole_super_groups():
    rng = np.random.default_rng(4)
    J = 12
    x = rng.standard_normal(J * 256).astype(f32)
    pos = rng.permutation(J).astype(np.uint32)
    out = P.reorder(x, pos)
    for j in range(J):
        assert np.array_equal(out[pos[j] * 256:(pos[j] + 1) * 256], x[j * 256:(j + 1) * 256])


def test_reorder_keeps_bf16_patterns():
    rng = np.random.default_rng(6)
    J = 6
    xb = rng.integers(0, 1 << 16, J * 256).astype(np.uint16)          # any pattern: the copy looks at no value
    pos = np.array([3, 0, 5, 1, 4, 2], np.uint32)
    out = P.reorder(xb, pos)
    for j in range(J):
        assert np.array_equal(out[pos[j] * 256:(pos[j] + 1) * 256], xb[j * 256:(j + 1) * 256])


def test_reorder_mean_follows_the_positions_and_zeroes_uncompressed_super_groups():
    w = np.array([8, 16, 2, 4, 16, 8, 2], np.uint8)
    mu = np.arange(1, 8, dtype=f32)                                    # mu[j] = j + 1
    pos, counts = P.positions(w)
    mm = P.reorder_mean(mu, pos, counts[3])
    # reordered order: the 2-bit ones (j = 2, 6), the 4-bit one (3), the 8-bit ones (0, 5), the 16-bit ones (1, 4)
    assert mm.tolist() == [3.0, 7.0, 4.0, 1.0, 6.0, 0.0, 0.0]
    assert P.reorder_mean(mu, pos, 0).tolist() == [3.0, 7.0, 4.0, 1.0, 6.0, 2.0, 5.0]


def test_restore_inverts_reorder_and_adds_n_mu():
    rng = np.random.default_rng(8)
    J, n = 9, 4
    # small integers times 2^-6: every sum and difference below is exact in fp32
    xs = [(rng.integers(-64, 64, J * 256) * 2.0 ** -6).astype(f32) for _ in range(n)]
    mu = (rng.integers(-8, 8, J) * 2.0 ** -6).astype(f32)
    w = rng.choice(np.array([2, 4, 8, 16], np.uint8), J)
    pos, counts = P.positions(w)
    mm = P.reorder_mean(mu, pos, counts[3])
    # what an exact main stage would return: the sum over workers of (entry - its mean), reordered
    total = sum(P.reorder(x, pos) for x in xs) - n * np.repeat(mm, 256)
    out = P.restore(total, pos, mm, n)
    assert np.array_equal(out, sum(xs))                     # sum_i (x_i - mu) + n mu = sum_i x_i
    kept = np.where(w == 16, f32(0), mu)                    # in the original order
    assert np.array_equal(P.restore(total, pos, None, n), sum(xs) - n * np.repeat(kept, 256))


def test_restore_without_means_is_the_permutation_alone():
    """Nothing subtracted, nothing added: every bit pattern survives, the sign of a zero included
    (x + 0.0 would turn -0.0 into +0.0)."""
    bits = np.arange(3 * 256, dtype=np.uint32) * np.uint32(0x00A3C0F1) | np.uint32(0x80000000)
    bits[:4] = [0x80000000, 0x00000000, 0x80000001, 0x7F7FFFFF]
    pos = np.array([2, 0, 1], np.uint32)
    out = P.restore(bits.view(f32), pos, None, 5)
    for j in range(3):
        assert np.array_equal(out[j * 256:(j + 1) * 256].view(np.uint32), bits[pos[j] * 256:(pos[j] + 1) * 256])


def test_pipeline_on_real_shapes():
    """statistics -> combine -> allocate -> positions on a bucket with the survey's structure."""
    rng = np.random.default_rng(10)
    n, J = 4, 512
    sig = np.exp(rng.normal(-7, 1.5, J))
    xs = [(rng.standard_normal((J, 256)) * sig[:, None]).astype(f32).reshape(-1) for _ in range(n)]
    st = [P.sg_stats(x) for x in xs]
    mu, F = P.stats_combine(np.array([s[0] for s in st], f32), np.array([s[1] for s in st], f32))
    F64 = sum(s[1] for s in st)
    assert np.allclose(F, F64, rtol=2.0 ** -7)              # bf16 contributions: 2^-9 each, relative
    budget = int(prep.code_bits(5.0) * J)
    w, _ = P.allocate(F, budget)
    assert budget - 6 < int(w.astype(int).sum()) <= budget  # the budget is used up to one step
    # larger norms never get fewer bits
    order = np.argsort(F, kind="stable")
    assert np.all(np.diff(w[order].astype(int)) >= 0)
