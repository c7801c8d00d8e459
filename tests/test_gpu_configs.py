"""The five benchmark configurations at FULL size, in the launch configuration bench.py times
(the hop replay), against the CPU oracle.

Configs 1-3: the oracle replays the whole schedule and every output entry is compared.
Configs 4-5: the GPU runs everything; the oracle recomputes sampled buckets (config 4) or
sampled runs of super-groups (config 5) one by one -- valid because a super-group's codes
depend only on its own data, its width and its global index.
"""
import numpy as np
import pytest
import torch

from oracle import dq_oracle as O
from paper_2602_08923_amd import binding as B
from paper_2602_08923_amd import prep, workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


def host(t):
    return t.detach().cpu().numpy()


def test_config2_ring8_bf16_25mb_full(dev):
    wl = workloads.CONFIGS[2]
    n = wl.n_workers
    grads = [workloads.draw(wl, w, 0, device="cpu") for w in range(n)]
    re, counts, perm = prep.prepare_bucket(grads, wl.budget_bits, n)
    n_sg = wl.entries // 256
    assert sum(counts) == n_sg and counts[0] > 0 and counts[1] > 0   # ~4 bits: a mix of 2- and 4-bit SGs
    seed = 2024
    mu = prep.mean_per_super_group(re)                                # as bench.py runs it: means subtracted
    trace = {}
    want = np.concatenate(O.ring_reduce_scatter(O.Oracle(n, seed=seed), [workloads.to_numpy(g) for g in re], counts,
                                                mu=mu.numpy(), trace=trace))
    ctx = B.Context(n, seed=seed)
    rp = B.Replay(ctx, B.DQ_RING, B.DQ_DYNAMIQ, [g.to(dev) for g in re], n_sg, [counts], mu=mu.to(dev))
    assert rp.n_steps == 8 and [rp.step_info(i)[0] for i in range(8)] == [0, 1, 1, 1, 1, 1, 1, 2]
    # every hop's packed message (codes, group scales, super-group scales) at full size, in the launch
    # shape the benchmark times: one step at a time, all 8 chunks of the step against the oracle's trace
    for t in range(n - 1):
        rp.run_steps(t, 1)
        torch.cuda.synchronize()
        for c in range(n):
            assert np.array_equal(host(rp.message(t, 0, c)), trace[(t, c)]), f"message of step {t}, chunk {c}"
    with pytest.raises(B.DqError):
        rp.message(n - 1, 0, 0)                                       # the last step writes sums, not a message
    rp.run_steps(n - 1, 1)
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out), want)
    rp.run()                                                          # and the whole schedule in one go, as timed
    torch.cuda.synchronize()
    got = host(rp.out)
    assert np.array_equal(got, want)
    true = sum(g.double() for g in re).numpy() - n * np.repeat(mu.double().numpy(), 256)
    assert ((got - true) ** 2).sum() / (true ** 2).sum() < 0.5   # ~4 bits, x100 outliers, 7 re-quantizations
    # the same bucket from the ORIGINAL tensors: super-groups gathered on the way in, scattered to
    # their original places with n * mu added on the way out -- restore(want) by definition
    from oracle import pp_oracle as P
    origin = perm.to(torch.int32).contiguous()                       # reordered[k] = original[perm[k]]
    pos = np.empty(n_sg, np.uint32)
    pos[perm.numpy()] = np.arange(n_sg, dtype=np.uint32)
    rg = B.Replay(ctx, B.DQ_RING, B.DQ_DYNAMIQ, [g.to(dev) for g in grads], n_sg, [counts], mu=mu.to(dev),
                  origin=origin.to(dev), inputs_in_original_order=True)
    rg.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rg.out).view(np.uint32), P.restore(want, pos, mu.numpy(), n).view(np.uint32))


@pytest.mark.parametrize("fmt", [B.DQ_MXFP8_E4M3, B.DQ_MXFP6_E3M2, B.DQ_MXFP4_E2M1])
def test_config3_ring8_mx_full(dev, fmt):
    wl = workloads.CONFIGS[3]
    n = wl.n_workers
    grads = [workloads.draw(wl, w, 0, device="cpu") for w in range(n)]
    want = np.concatenate(O.mx_ring_reduce_scatter(fmt, [workloads.to_numpy(g) for g in grads]))
    ctx = B.Context(n)
    rp = B.Replay(ctx, B.DQ_RING, fmt, [g.to(dev) for g in grads], wl.entries // 256)
    rp.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out), want)


def test_config4_butterfly16_1p3b_sampled_buckets(dev):
    """16-worker butterfly over 100 buckets of 13,107,200 bf16 entries (1.31 B parameters per
    worker, 42 GB of gradients in HBM), b = 3; the oracle recomputes five whole buckets."""
    wl = workloads.CONFIGS[4]
    n, d, nb = wl.n_workers, wl.entries, wl.n_buckets
    n_sg = d // 256
    check = (0, 7, 41, 93, 99)
    worker = [torch.empty(d * nb, dtype=torch.bfloat16, device=dev) for _ in range(n)]
    counts_all, kept, mus = [], {}, []
    for b in range(nb):
        g = [workloads.draw(wl, w, b, device=dev) for w in range(n)]
        re, counts, _ = prep.prepare_bucket(g, wl.budget_bits, n)
        counts_all.append(counts)
        mus.append(prep.mean_per_super_group(re))
        for w in range(n):
            worker[w][b * d:(b + 1) * d] = re[w]
        if b in check:
            kept[b] = [workloads.to_numpy(x) for x in re]
        del g, re
    assert len({tuple(c) for c in counts_all}) > 2      # buckets that straddle two tensors get other allocations
    assert all(c[0] > 0 for c in counts_all)            # lowest budget: mostly 2-bit
    seed = 77
    ctx = B.Context(n, seed=seed)
    rp = B.Replay(ctx, B.DQ_BUTTERFLY, B.DQ_DYNAMIQ, worker, n_sg, counts_all, n_buckets=nb, mu=torch.cat(mus))
    assert rp.n_steps == 5
    rp.run()
    torch.cuda.synchronize()
    orc = O.Oracle(n, seed=seed)
    for b in check:
        want = np.concatenate(O.butterfly_reduce_scatter(orc, kept[b], counts_all[b], first_sg=b * n_sg,
                                                         mu=mus[b].cpu().numpy()))
        got = host(rp.out[b * d:(b + 1) * d])
        assert np.array_equal(got, want), f"bucket {b}"
    # the unchecked buckets are estimates of their true sums too (at 3 bits per entry on i.i.d.
    # values the ternary codes are coarse: ask for clear correlation, not for a small error)
    for b in (0, 50, 99):
        true = sum(worker[w][b * d:(b + 1) * d].double() for w in range(n)) - n * mus[b].double().repeat_interleave(256)
        est = rp.out[b * d:(b + 1) * d].double()
        corr = float((est * true).sum() / torch.sqrt((est * est).sum() * (true * true).sum()))
        assert corr > 0.5, (b, corr)


def test_config5_chain64_125m_sampled_runs(dev):
    """One chunk of a 64-worker ring: 64 slices of 125,000,192 bf16 entries (16 GB), all 63 hops
    replayed with the packed partial sums kept in HBM; the oracle recomputes sampled runs."""
    wl = workloads.CONFIGS[5]
    n, d = wl.n_workers, wl.entries
    n_sg = d // 256
    F = None
    raw = []
    for w in range(n):
        g = workloads.draw(wl, w, 0, device=dev)
        f = g.to(torch.float64).reshape(-1, 256).pow(2).sum(dim=1)
        F = f if F is None else F + f
        raw.append(g)
    widths = prep.allocate(F, wl.budget_bits)
    perm, counts = prep.reorder_plan(widths, 1)
    del F, widths
    slices = []
    for w in range(n):
        slices.append(prep.apply_reorder(raw[w], perm))
        raw[w] = None
    assert counts[1] > 0 and counts[2] > 0              # 4.3125 code bits on average: 4- and 8-bit SGs
    seed = 5
    mu = prep.mean_per_super_group(slices)
    ctx = B.Context(n, seed=seed)
    rp = B.Replay(ctx, B.DQ_CHAIN, B.DQ_DYNAMIQ, slices, n_sg, [counts], mu=mu)
    assert rp.n_steps == 64
    assert [rp.step_info(i)[0] for i in (0, 1, 62, 63)] == [0, 1, 1, 2]
    rp.run()
    torch.cuda.synchronize()
    # sampled runs: the start, both width boundaries (runs that straddle them), the ragged end
    edges = np.cumsum([0] + counts)
    run = 96
    starts = [0, int(edges[1]) - 40, int(edges[1]) + 1000, int(edges[2]) - 50, (n_sg // 2 // 4) * 4 + 1, n_sg - run]
    orc = O.Oracle(n, seed=seed)
    # ... and 40 longer runs at seeded random places (with the six above about 2 % of the chunk)
    rng = np.random.default_rng(2602)
    sampled = [(s, run) for s in starts] + [(int(s), 256) for s in rng.integers(0, n_sg - 256, 40)]
    for s, run in sampled:
        s = max(0, min(s, n_sg - run))
        cw = [int(max(0, min(s + run, edges[k + 1]) - max(s, edges[k]))) for k in range(3)]
        ch = O.make_chunk(s, cw)
        sl = [workloads.to_numpy(x[s * 256:(s + run) * 256]) for x in slices]
        m = mu[s:s + run].cpu().numpy()
        msg = orc.compress(ch, 0, sl[0], m)
        for i in range(1, n - 1):
            msg = orc.dar_hop(ch, i, msg, sl[i], m)
        want = orc.decompress(ch, msg, sl[n - 1], m)
        got = host(rp.out[s * 256:(s + run) * 256])
        assert np.array_equal(got, want), f"run at super-group {s}"


def test_one_chunk_beyond_four_gibibytes(dev):
    """A single chunk of 20.5 M super-groups (5.2 G entries): the local slice (10.5 GB), the 8-bit
    codes (4.5 GB), the entry index and the fp32 result (21 GB) all pass 2^32 inside one job, so every
    64-bit offset of the kernels is exercised.  Compress, a DAR hop and decompress-accumulate run at
    full size; the oracle recomputes runs of super-groups around each 2^32 crossing, the width
    boundaries and the ragged end."""
    free, _ = torch.cuda.mem_get_info()
    if free < 60 * 2 ** 30:
        pytest.skip("needs 60 GB of free device memory")
    n = 8
    counts = [1_000_003, 2_000_001, 17_500_002]                  # not multiples of a tile: ragged segment ends
    n_sg = sum(counts)
    entries = n_sg * 256
    local = torch.empty(entries, dtype=torch.bfloat16, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(20260208)
    step = 1 << 28
    for lo in range(0, entries, step):                           # sigma varies slowly along the tensor
        hi = min(entries, lo + step)
        x = torch.randn(hi - lo, generator=gen, device=dev) * (1e-3 * (1 + lo / entries))
        local[lo:hi] = x.to(torch.bfloat16)
        del x
    mu = (torch.randn(n_sg, generator=gen, device=dev) * 1e-5).contiguous()
    first = 3
    seed = 99
    ctx = B.Context(n, seed=seed)
    gch = B.make_chunk(first, counts)
    p1 = ctx.dq_compress(local, gch, 2, mu=mu)
    p2 = ctx.dq_dar_hop(p1, local, gch, 5, mu=mu)
    out = ctx.dq_decompress(p2, gch, local=local, mu=mu)
    torch.cuda.synchronize()
    edges = np.cumsum([0] + counts)
    run = 96
    code8_cross = int(edges[2]) + (2 ** 32 - 64 * counts[0] - 128 * counts[1]) // 256   # 8-bit code bytes pass 2^32 here
    starts = [0, int(edges[1]) - 50, int(edges[2]) - 47, 2 ** 22 - 40, 2 ** 23 - 48, 2 ** 24 - 50, code8_cross - 45,
              n_sg - run]
    assert all(0 <= s <= n_sg - run for s in starts) and code8_cross < n_sg
    orc = O.Oracle(n, seed=seed)
    for s in starts:
        cw = [int(max(0, min(s + run, edges[k + 1]) - max(s, edges[k]))) for k in range(3)]
        ch = O.make_chunk(first + s, cw)
        sl = workloads.to_numpy(local[s * 256:(s + run) * 256].cpu())
        m = mu[s:s + run].cpu().numpy()
        msg = orc.dar_hop(ch, 5, orc.compress(ch, 2, sl, m), sl, m)
        want = orc.decompress(ch, msg, sl, m)
        assert np.array_equal(host(out[s * 256:(s + run) * 256]).view(np.uint32), want.view(np.uint32)), f"run at super-group {s}"


def test_mx_beyond_four_gibibytes(dev):
    """The MX codec on 5.2 G entries in one call (codes, local bytes, entry index and result pass 2^32)."""
    free, _ = torch.cuda.mem_get_info()
    if free < 60 * 2 ** 30:
        pytest.skip("needs 60 GB of free device memory")
    fmt = B.DQ_MXFP8_E4M3
    entries = (2 ** 32 + 2 ** 30 + 7 * 256)
    local = torch.empty(entries, dtype=torch.bfloat16, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    step = 1 << 28
    for lo in range(0, entries, step):
        hi = min(entries, lo + step)
        local[lo:hi] = (torch.randn(hi - lo, generator=gen, device=dev) * 1e-3).to(torch.bfloat16)
    p2 = B.dq_mx_dar_hop(fmt, B.dq_mx_compress(fmt, local), local)
    out = B.dq_mx_decompress(fmt, p2, entries, local=local)
    torch.cuda.synchronize()
    run = 4096
    for s in (0, 2 ** 30 - 2048, 2 ** 31 - 2048, 2 ** 32 - 2048, entries - run):
        sl = workloads.to_numpy(local[s:s + run].cpu())
        want = O.mx_decompress(fmt, O.mx_dar_hop(fmt, O.mx_compress(fmt, sl), sl), run, sl)
        assert np.array_equal(host(out[s:s + run]).view(np.uint32), want.view(np.uint32)), f"run at entry {s}"
