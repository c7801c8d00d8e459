"""HIP path of the steps before and after the main stage against the CPU oracle
(oracle/pp_oracle.c), through the C ABI.  Each stage gets the oracle's output of the stage
before it (never the other way round): statistics within the tolerance of fp32 accumulation
against the float64 definition, everything that is an integer decision or a single rounded
operation bit-exactly."""
import math

import numpy as np
import pytest
import torch

from oracle import pp_oracle as P
from paper_2602_08923_amd import binding as B
from paper_2602_08923_amd import prep, workloads

pytestmark = pytest.mark.gpu
f32 = np.float32


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


def host(t):
    return t.detach().cpu().numpy()


def draw(cfg, worker, entries, bucket=0):
    return workloads.draw(workloads.CONFIGS[cfg], worker, bucket, device="cpu", entries=entries)


def as_np(t):
    return workloads.to_numpy(t)


def lognormal_F(seed, J, zeros=0, ties=0):
    rng = np.random.default_rng(seed)
    F = np.exp(rng.normal(-14, 2.5, J)).astype(f32)
    if zeros:
        F[rng.integers(0, J, zeros)] = 0
    if ties:
        F[rng.integers(0, J, ties)] = F[0]
    return F


# ---------------------------------------------------------------- statistics
@pytest.mark.parametrize("cfg,n_sg", [(1, 1), (1, 5), (2, 1027), (4, 4096), (5, 2049)])
def test_sg_stats(dev, cfg, n_sg):
    x = draw(cfg, 3, n_sg * 256)
    mu64, F64 = P.sg_stats(as_np(x))
    mu, F = B.dq_sg_stats(x.to(dev))
    mu, F = host(mu).astype(np.float64), host(F).astype(np.float64)
    # 16 sequential + 4 tree additions in fp32: relative error below 20 * 2^-24 of the sum of magnitudes
    tol = 20 * 2.0 ** -24
    assert np.all(np.abs(F - F64) <= tol * F64 + 1e-45)
    mean_abs = np.abs(x.double().numpy().reshape(n_sg, 256)).sum(axis=1) / 256
    assert np.all(np.abs(mu - mu64) <= tol * mean_abs + 1e-45)
    assert np.all(F64 > 0)


def test_sg_stats_exact_cases(dev):
    c = 0.375
    x = np.concatenate([np.full(256, c), np.tile([0.5, -0.5], 128), np.arange(256) * 2.0 ** -10, np.zeros(256)]).astype(f32)
    for t in (torch.from_numpy(x), torch.from_numpy(x).to(torch.bfloat16)):      # all values are bf16-exact
        mu, F = B.dq_sg_stats(t.to(dev))
        assert host(mu).tolist() == [c, 0.0, 127.5 * 2.0 ** -10, 0.0]
        assert host(F).tolist() == [256 * c * c, 64.0, 5559680 * 2.0 ** -20, 0.0]
    mu, F = B.dq_sg_stats(torch.empty(0, dtype=torch.float32, device=dev))       # empty input
    assert mu.numel() == 0 and F.numel() == 0


def test_stats_combine(dev):
    n, J = 8, 3001
    xs = [draw(2, w, J * 256) for w in range(n)]
    st = [P.sg_stats(as_np(x)) for x in xs]
    mu_all = np.array([s[0] for s in st], f32)
    F_all = np.array([s[1] for s in st], f32)
    want_mu, want_F = P.stats_combine(mu_all, F_all)
    mu, F = B.dq_stats_combine(torch.from_numpy(mu_all).to(dev), torch.from_numpy(F_all).to(dev))
    assert np.array_equal(host(mu).view(np.uint32), want_mu.view(np.uint32))
    assert np.array_equal(host(F).view(np.uint32), want_F.view(np.uint32))
    # n = 1 and a worker count that is not a power of two (the division is rounded, not a shift)
    for k in (1, 3):
        want_mu, want_F = P.stats_combine(mu_all[:k], F_all[:k])
        mu, F = B.dq_stats_combine(torch.from_numpy(mu_all[:k].copy()).to(dev), torch.from_numpy(F_all[:k].copy()).to(dev))
        assert np.array_equal(host(mu).view(np.uint32), want_mu.view(np.uint32))
        assert np.array_equal(host(F).view(np.uint32), want_F.view(np.uint32))


# ---------------------------------------------------------------- allocation
def check_allocate(dev, F, J, budget, max_width=8):
    nb = F.size // J
    widths, pos, counts = B.dq_allocate(torch.from_numpy(F).to(dev), J, budget, max_width=max_width)
    widths, pos, counts = host(widths), host(pos).view(np.uint32), host(counts).view(np.uint32)
    for b in range(nb):
        w, tbits = P.allocate(F[b * J:(b + 1) * J], budget, max_width=max_width)
        p, c = P.positions(w)
        assert np.array_equal(widths[b * J:(b + 1) * J], w), f"bucket {b}"
        assert np.array_equal(pos[b * J:(b + 1) * J], p), f"bucket {b}"
        assert counts[b].tolist() == c + [tbits], f"bucket {b}"
    return counts


@pytest.mark.parametrize("J", [1, 7, 64, 1000, 1024, 1025, 51200, 65536])
@pytest.mark.parametrize("bits", [3.0, 5.0])
def test_allocate_sizes(dev, J, bits):
    F = lognormal_F(J, J, zeros=min(J // 10, 50), ties=min(J // 7, 40))
    check_allocate(dev, F, J, int(math.floor(prep.code_bits(bits) * J)))


@pytest.mark.parametrize("J", [1, 64, 1025, 51200, 70000])
@pytest.mark.parametrize("bits", [5.0, 8.5, 12.0])
def test_allocate_with_sixteen_bit_class(dev, J, bits):
    F = lognormal_F(J + 1, J, zeros=min(J // 10, 50), ties=min(J // 7, 40))
    c = check_allocate(dev, F, J, int(math.floor(prep.code_bits(bits) * J)), max_width=16)
    if J >= 1025 and bits >= 8.5:
        assert c[0][3] > 0                       # some super-groups do get 16 bits


def test_allocate_many_buckets_full_size(dev):
    """config 4's shape: 100 buckets of 51,200 super-groups, one block per bucket."""
    J, nb = 51200, 100
    rng = np.random.default_rng(4)
    F = np.concatenate([np.exp(rng.normal(rng.uniform(-20, -8), rng.uniform(0.5, 3.0), J)) for _ in range(nb)]).astype(f32)
    counts = check_allocate(dev, F, J, int(math.floor(prep.code_bits(3.0) * J)))
    assert len({tuple(c[:3]) for c in counts.tolist()}) > 50


def test_allocate_beyond_register_capacity(dev):
    J = 65536 + 4321                                   # runs no longer fit 64 registers per thread
    F = lognormal_F(99, 2 * J, zeros=100, ties=100)
    check_allocate(dev, F, J, int(math.floor(prep.code_bits(4.0) * J)))


@pytest.mark.parametrize("bits", [2.8, 4.0, 6.0, 8.5])
def test_allocate_masses_of_equal_values(dev, bits):
    """More equal norms than the kernel keeps as candidates of its narrowed search: it must fall
    back to counting everything and still agree."""
    J = 51200
    F = lognormal_F(21, J)
    F[5000:35000] = F[7]                      # 30,000 equal values
    F[40000:46000] = np.float32(F[7] * np.float32(17.0 / 512.0))   # and 6,000 at the tied lower threshold
    check_allocate(dev, F, J, int(math.floor(prep.code_bits(bits) * J)))
    check_allocate(dev, np.full(J, 3.25e-7, f32), J, int(math.floor(prep.code_bits(bits) * J)))


def test_allocate_narrow_value_ranges(dev):
    """Norms one bit pattern apart around the threshold, two distinct values tied by the threshold
    ratio, several small buckets per call."""
    J = 20000
    base = np.float32(1.5e-3)
    pat = base.view(np.uint32) + np.arange(J, dtype=np.uint32) % 300          # 300 neighbouring patterns
    F = pat.view(f32).copy()
    for bits in (2.8, 4.0, 7.0):
        check_allocate(dev, F, J, int(math.floor(prep.code_bits(bits) * J)))
    F2 = np.where(np.arange(J) % 3 == 0, np.float32(2.0), np.float32(2.0 * 17.0 / 512.0)).astype(f32)
    for bits in (2.8, 3.5, 4.0, 6.0):
        check_allocate(dev, F2, J, int(math.floor(prep.code_bits(bits) * J)))
        check_allocate(dev, F2, J, int(math.floor(prep.code_bits(bits) * J)), max_width=16)
    F3 = lognormal_F(8, 3 * 4097)
    check_allocate(dev, F3, 4097, int(math.floor(prep.code_bits(4.0) * 4097)))   # 3 buckets, 5 rows each, ragged


def test_allocate_more_buckets_than_a_grid_dimension(dev):
    """70,000 buckets of 5 super-groups: the positions launch is cut at 65,535 buckets (the grid's second
    dimension); buckets on both sides of the cut must come out right."""
    J, nb = 5, 70000
    F = lognormal_F(17, J * nb)
    budget = 4 * J + 2
    widths, pos, counts = B.dq_allocate(torch.from_numpy(F).to(dev), J, budget)
    widths, pos, counts = host(widths), host(pos).view(np.uint32), host(counts).view(np.uint32)
    for b in list(range(0, nb, 997)) + [65534, 65535, 65536, nb - 1]:
        w, tbits = P.allocate(F[b * J:(b + 1) * J], budget)
        p, c = P.positions(w)
        assert np.array_equal(widths[b * J:(b + 1) * J], w), f"bucket {b}"
        assert np.array_equal(pos[b * J:(b + 1) * J], p), f"bucket {b}"
        assert counts[b].tolist() == c + [tbits], f"bucket {b}"


def test_allocate_budget_edges(dev):
    F = lognormal_F(5, 2000)
    c = check_allocate(dev, F, 2000, 2 * 2000)                       # exactly 2 bits each
    assert c[0][:3].tolist() == [2000, 0, 0]
    c = check_allocate(dev, F, 2000, 8 * 2000 + 5)                   # everything fits
    assert c[0][:3].tolist() == [0, 0, 2000] and c[0][4] == 1
    c = check_allocate(dev, np.zeros(512, f32), 512, 3 * 512)        # an all-zero bucket
    assert c[0][:3].tolist() == [512, 0, 0]
    with pytest.raises(B.DqError):
        B.dq_allocate(torch.from_numpy(F).to(dev), 2000, 3999)       # below 2 bits per coordinate


# ---------------------------------------------------------------- reorder / restore
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("J,nb", [(1, 1), (37, 3), (1030, 2)])
def test_reorder_and_restore(dev, dtype, J, nb):
    n_sg = J * nb
    x = draw(2 if dtype == "bf16" else 1, 1, n_sg * 256)
    rng = np.random.default_rng(J)
    widths = rng.choice(np.array([2, 4, 8, 16], np.uint8), n_sg, p=[0.4, 0.3, 0.2, 0.1])
    pc = [P.positions(widths[b * J:(b + 1) * J]) for b in range(nb)]
    pos = np.concatenate([p for p, _ in pc])
    counts = np.array([c + [0] for _, c in pc], np.int32)                  # [nb, 5] as dq_allocate writes it
    mu = (rng.standard_normal(n_sg) * 1e-4).astype(f32)
    xn = as_np(x)
    pos_t = torch.from_numpy(pos.view(np.int32)).to(dev)
    want = np.concatenate([P.reorder(xn[b * J * 256:(b + 1) * J * 256], pos[b * J:(b + 1) * J]) for b in range(nb)])
    got = B.dq_reorder(x.to(dev), pos_t, J)
    assert np.array_equal(as_np(got.cpu()), want)
    # the means of the main stage: reordered, zero for the 16-bit super-groups; without counts: all kept
    for cnt in (counts, None):
        want_mm = np.concatenate([P.reorder_mean(mu[b * J:(b + 1) * J], pos[b * J:(b + 1) * J],
                                                 0 if cnt is None else cnt[b][3]) for b in range(nb)])
        got_mm = B.dq_reorder_mean(torch.from_numpy(mu).to(dev), pos_t, J,
                                   None if cnt is None else torch.from_numpy(cnt).to(dev))
        assert np.array_equal(host(got_mm).view(np.uint32), want_mm.view(np.uint32))
    # the inverse of the positions, alone and together with the means
    inv = np.concatenate([np.argsort(pos[b * J:(b + 1) * J]) for b in range(nb)]).astype(np.int32)
    _, origin = B.dq_reorder_mean(None, pos_t, J, with_origin=True)
    assert np.array_equal(host(origin), inv)
    mm2, origin2 = B.dq_reorder_mean(torch.from_numpy(mu).to(dev), pos_t, J, with_origin=True)
    assert np.array_equal(host(origin2), inv) and np.array_equal(host(mm2).view(np.uint32), want_mm.view(np.uint32))
    total = (rng.standard_normal(n_sg * 256) * 1e-2).astype(f32)
    for m in (want_mm, None):
        want = np.concatenate([P.restore(total[b * J * 256:(b + 1) * J * 256], pos[b * J:(b + 1) * J],
                                         None if m is None else m[b * J:(b + 1) * J], 8) for b in range(nb)])
        got = B.dq_restore(torch.from_numpy(total).to(dev), pos_t, J, 8,
                           mu_main=None if m is None else torch.from_numpy(m).to(dev))
        assert np.array_equal(host(got).view(np.uint32), want.view(np.uint32))


def test_reorder_full_bucket(dev):
    """One worker's whole config-2 bucket (13,107,200 bf16 entries), allocation from the oracle."""
    wl = workloads.CONFIGS[2]
    J = wl.entries // 256
    x = workloads.draw(wl, 0, 0, device="cpu")
    mu64, F64 = P.sg_stats(as_np(x))
    mu, F = P.stats_combine(mu64.astype(f32)[None], (8 * F64).astype(f32)[None])
    w, _ = P.allocate(F, int(math.floor(prep.code_bits(wl.budget_bits) * J)))
    pos, counts = P.positions(w)
    assert counts[0] > 0 and counts[1] > 0
    pos_t = torch.from_numpy(pos.view(np.int32)).to(dev)
    got = B.dq_reorder(x.to(dev), pos_t, J)
    assert np.array_equal(as_np(got.cpu()), P.reorder(as_np(x), pos))
    mm = P.reorder_mean(mu, pos, 0)
    got_mm = B.dq_reorder_mean(torch.from_numpy(mu).to(dev), pos_t, J)
    assert np.array_equal(host(got_mm).view(np.uint32), mm.view(np.uint32))
    total = got.float()
    back = B.dq_restore(total, pos_t, J, 1, mu_main=got_mm)
    assert np.array_equal(host(back).view(np.uint32), P.restore(host(total), pos, mm, 1).view(np.uint32))
    # the permutation alone is undone exactly
    assert torch.equal(B.dq_restore(total, pos_t, J, 1).cpu(), x.float())


def test_rejects_bad_arguments(dev):
    x = torch.zeros(512, dtype=torch.float32, device=dev)
    pos = torch.zeros(2, dtype=torch.int32, device=dev)
    L = B.lib()
    st = L.dq_reorder(B._ptr(x), 0, B._ptr(pos), 2, 1, B._ptr(x), None)               # in place
    assert st == B.DQ_EINVAL
    st = L.dq_reorder(x.data_ptr() + 4, 0, B._ptr(pos), 2, 1, B._ptr(torch.empty_like(x)), None)
    assert st == B.DQ_EALIGN
    mu = torch.zeros(2, dtype=torch.float32, device=dev)
    st = L.dq_reorder_mean(B._ptr(mu), B._ptr(pos), None, 2, 1, B._ptr(mu), None, None)     # in place
    assert st == B.DQ_EINVAL
    st = L.dq_reorder_mean(B._ptr(mu), B._ptr(pos), None, 2, 1, None, None, None)           # no output asked for
    assert st == B.DQ_EINVAL
    st = L.dq_restore(B._ptr(x), B._ptr(pos), None, 0, 2, 1, B._ptr(torch.empty_like(x)), None)   # n = 0
    assert st == B.DQ_EINVAL
    st = L.dq_sg_stats(B._ptr(x), 7, 2, B._ptr(x), B._ptr(x), None)                  # unknown dtype
    assert st == B.DQ_EINVAL


def test_whole_pipeline_is_consistent(dev):
    """statistics -> combine -> allocate -> reorder -> ring reduce-scatter -> restore, all on the GPU:
    the allocation meets its budget with larger norms never getting fewer bits, and the restored
    result estimates the true sum."""
    wl = workloads.CONFIGS[2]
    n, J = 8, 4096
    xs = [workloads.draw(wl, w, 0, device=dev, entries=J * 256) for w in range(n)]
    xs[3][:256] += 0.5                                                   # a super-group with a large mean
    st = [B.dq_sg_stats(x) for x in xs]
    mu, F = B.dq_stats_combine(torch.stack([s[0] for s in st]), torch.stack([s[1] for s in st]))
    budget = int(math.floor(prep.code_bits(5.0) * J))
    widths, pos, counts = B.dq_allocate(F, J, budget)
    c = counts.cpu().numpy()[0]
    w = host(widths).astype(int)
    assert sum(c[:4]) == J and budget - 6 < int(w.sum()) <= budget
    order = np.argsort(host(F), kind="stable")
    assert np.all(np.diff(w[order]) >= 0)
    re = [B.dq_reorder(x, pos, J) for x in xs]
    mu_main = B.dq_reorder_mean(mu, pos, J, counts)
    ctx = B.Context(n, seed=11)
    rp = B.Replay(ctx, B.DQ_RING, B.DQ_DYNAMIQ, re, J, [[int(v) for v in c[:3]]], mu=mu_main)
    rp.run()
    out = B.dq_restore(rp.out, pos, J, n, mu_main=mu_main)
    true = sum(x.double() for x in xs)
    est = out.double()
    assert float(((est - true) ** 2).sum() / (true ** 2).sum()) < 0.05
    # the shifted super-group: without the mean handling its 0.5 offset would dominate the error
    assert float((est[:256] - true[:256]).abs().max()) < 0.02
