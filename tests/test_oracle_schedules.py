"""The oracle's hop schedules (Section 3.4, Appendix B) against plain definitions."""
import numpy as np
import pytest

from oracle import dq_oracle as O


def grads(n, n_sg, seed, dtype=np.float32):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        g = (rng.standard_normal(n_sg * 256) * 1e-3).astype(np.float32)
        if dtype == np.uint16:
            g = (g.view(np.uint32) >> 16).astype(np.uint16)
        out.append(g)
    return out


def widen(g):
    return g if g.dtype == np.float32 else (g.astype(np.uint32) << 16).view(np.float32)


def vnmse(out, gs):
    s = sum(widen(g).astype(np.float64) for g in gs)
    e = np.concatenate(out).astype(np.float64) - s
    return float((e ** 2).sum() / (s ** 2).sum())


def test_split_bucket_covers_every_super_group_once():
    chunks = O.split_bucket([5, 9, 2], 4, first_sg=100)
    assert [c.first_sg for c in chunks] == [100, 104, 108, 112]
    assert [list(c.n_sg) for c in chunks] == [[4, 0, 0, 0], [1, 3, 0, 0], [0, 4, 0, 0], [0, 2, 2, 0]]
    chunks = O.split_bucket([2, 1, 2, 3], 4)                      # with a run of 16-bit super-groups
    assert [list(c.n_sg) for c in chunks] == [[2, 0, 0, 0], [0, 1, 1, 0], [0, 0, 1, 1], [0, 0, 0, 2]]
    with pytest.raises(AssertionError):
        O.split_bucket([5, 9, 1], 4)


def test_ring_two_workers_is_compress_then_decompress_add():
    orc = O.Oracle(2, seed=3)
    gs = grads(2, 4, 1)
    out = O.ring_reduce_scatter(orc, gs, [0, 4, 0])
    chunks = O.split_bucket([0, 4, 0], 2)
    for c in range(2):
        sl = slice(c * 512, (c + 1) * 512)
        msg = orc.compress(chunks[c], c, gs[c][sl])
        want = orc.decompress(chunks[c], msg, gs[(c + 1) % 2][sl])
        assert np.array_equal(out[c], want)


def test_ring_trace_and_ranks():
    """Chunk c is compressed by worker c, re-encoded by c+1..c+n-2, finished by c+n-1."""
    n = 4
    orc = O.Oracle(n, seed=5)
    gs = grads(n, 8, 2)
    trace = {}
    out = O.ring_reduce_scatter(orc, gs, [2, 4, 2], trace=trace)
    chunks = O.split_bucket([2, 4, 2], n)
    for c in range(n):
        sl = slice(c * 512, (c + 1) * 512)
        msg = orc.compress(chunks[c], c, gs[c][sl])
        assert np.array_equal(trace[(0, c)], msg)
        for t in (1, 2):
            msg = orc.dar_hop(chunks[c], (c + t) % n, msg, gs[(c + t) % n][sl])
            assert np.array_equal(trace[(t, c)], msg)
        assert np.array_equal(out[c], orc.decompress(chunks[c], msg, gs[(c + 3) % n][sl]))


@pytest.mark.parametrize("dtype", [np.float32, np.uint16])
def test_reduce_scatter_approximates_the_sum(dtype):
    n = 8
    orc = O.Oracle(n, seed=7)
    gs = grads(n, 16, 3, dtype)
    e8 = vnmse(O.ring_reduce_scatter(orc, gs, [0, 0, 16]), gs)
    e4 = vnmse(O.ring_reduce_scatter(orc, gs, [0, 16, 0]), gs)
    e2 = vnmse(O.ring_reduce_scatter(orc, gs, [16, 0, 0]), gs)
    assert e8 < 1e-3 and e8 < e4 < e2
    b4 = vnmse(O.butterfly_reduce_scatter(orc, gs, [0, 16, 0]), gs)
    assert b4 < e4  # shorter aggregation paths re-quantize less often (Appendix B)


def test_butterfly_two_workers_equals_ring_two_workers():
    orc = O.Oracle(2, seed=11)
    gs = grads(2, 4, 4)
    ring = O.ring_reduce_scatter(orc, gs, [1, 2, 1])
    bfly = O.butterfly_reduce_scatter(orc, gs, [1, 2, 1])
    # ring: chunk c is compressed by worker c and ends at worker c+1; butterfly: worker w keeps
    # chunk w and receives it compressed by w^1.  Same pairs, opposite roles.
    chunks = O.split_bucket([1, 2, 1], 2)
    for w in range(2):
        sl = slice(w * 512, (w + 1) * 512)
        msg = orc.compress(chunks[w], w ^ 1, gs[w ^ 1][sl])
        assert np.array_equal(bfly[w], orc.decompress(chunks[w], msg, gs[w][sl]))
    assert len(ring) == len(bfly) == 2


def test_butterfly_four_workers_by_hand():
    """n = 4: step 1 exchanges halves with w^2, step 2 quarters with w^1 (Appendix B)."""
    n = 4
    orc = O.Oracle(n, seed=13)
    gs = grads(n, 8, 5)
    ch = O.split_bucket([0, 8, 0], n)
    m = 512

    def sl(c):
        return slice(c * m, (c + 1) * m)

    out = O.butterfly_reduce_scatter(orc, gs, [0, 8, 0])
    # worker 0 ends with chunk 0.  Step 1: worker 2 sends compress(chunks 0,1) to worker 0.
    # Step 2: worker 1 (which got chunks 0,1 from worker 3) re-encodes chunk 0 for worker 0.
    m_3to1 = orc.compress(ch[0], 3, gs[3][sl(0)])
    m_1to0 = orc.dar_hop(ch[0], 1, m_3to1, gs[1][sl(0)])
    m_2to0 = orc.compress(ch[0], 2, gs[2][sl(0)])
    acc0 = orc.decompress(ch[0], m_2to0, gs[0][sl(0)])
    want = orc.decompress(ch[0], m_1to0, acc0)
    assert np.array_equal(out[0], want)


def test_single_worker_passthrough():
    orc = O.Oracle(1)
    gs = grads(1, 2, 6)
    out = O.ring_reduce_scatter(orc, gs, [0, 2, 0])
    assert np.array_equal(out[0], gs[0])


# ----------------------------------------------------------------- all-gather phase (Section 3.4)

def test_all_gather_is_compress_then_decompress_by_the_sink():
    """Chunk c's sum is compressed by the worker where its reduce-scatter ended (ring: c-1 mod n,
    recursive halving: c) and everyone keeps the decompressed message."""
    n = 4
    orc = O.Oracle(n, seed=3)
    counts = [4, 8, 4]
    rng = np.random.default_rng(1)
    sums = [(rng.standard_normal(4 * 256) * 1e-2).astype(np.float32) for _ in range(n)]
    chunks = O.split_bucket(counts, n, first_sg=40)
    for topo, sink_of in (("ring", lambda c: (c - 1) % n), ("butterfly", lambda c: c)):
        got = O.all_gather(orc, sums, counts, topo, first_sg=40)
        for c in range(n):
            want = orc.decompress(chunks[c], orc.compress(chunks[c], sink_of(c), sums[c]))
            assert np.array_equal(got[c], want)
            other = orc.decompress(chunks[c], orc.compress(chunks[c], (sink_of(c) + 1) % n, sums[c]))
            assert not np.array_equal(got[c], other)          # the rank feeds the rounding


def test_all_gather_keeps_lattice_values_and_estimates_the_rest():
    n = 4
    orc = O.Oracle(n, seed=8)
    T = orc.T(1)
    rng = np.random.default_rng(2)
    r = rng.integers(0, 8, 4 * 256)
    r[::16] = 7
    lattice = (np.where(rng.integers(0, 2, r.size) == 1, -1.0, 1.0) * T[r].astype(np.float64) * 0.5).astype(np.float32)
    counts = [0, 4, 0]                                         # four 4-bit super-groups, one per chunk
    sums = [lattice[c * 256:(c + 1) * 256] for c in range(n)]
    out = O.all_gather(orc, sums, counts, "ring")
    for c in range(n):
        nz = sums[c] != 0
        assert np.array_equal(out[c][nz], sums[c][nz])         # values on the codec's lattice survive
    # off the lattice: every entry lands within one level gap of its group's scale
    rough = [(rng.standard_normal(256) * 1e-3).astype(np.float32) for _ in range(n)]
    out = O.all_gather(orc, rough, counts, "butterfly")
    for c in range(n):
        g = np.abs(rough[c]).reshape(16, 16).max(axis=1)
        bound = np.repeat(g, 16) * (float(T[7] - T[6]) + 1.0 / 255 + 2.0 ** -7)
        assert np.all(np.abs(out[c] - rough[c]) <= bound)


# ----------------------------------------------------------------- 16-bit (uncompressed) super-groups

def test_sixteen_bit_super_groups_travel_as_bf16():
    """Section 3.2: "16 bits corresponds to uncompressed values".  Such a super-group is 256 raw
    bf16 numbers: no scales, no randomness; every hop adds in fp32 and rounds to bf16."""
    import torch
    n = 4
    orc = O.Oracle(n, seed=1)
    rng = np.random.default_rng(5)
    ch = O.make_chunk(7, [1, 2, 1, 3])
    assert O.Oracle.packed_bytes(ch) == 64 + 2 * 128 + 256 + 3 * 512 + 4 * 18 + 8     # scales for the 4 coded SGs, padded to 16
    x = (rng.standard_normal(7 * 256) * 1e-2).astype(np.float32)
    y = (rng.standard_normal(7 * 256) * 1e-2).astype(np.float32)
    msg = orc.compress(ch, 0, x)
    raw = msg[64 + 256 + 256:64 + 256 + 256 + 3 * 512].view(np.uint16)
    want = torch.from_numpy(x[4 * 256:]).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(raw, want)                                   # the values themselves, rounded to nearest even
    # independent of rank and seed: nothing random in it
    other = O.Oracle(n, seed=99).compress(ch, 3, x)
    assert np.array_equal(other[64 + 512:64 + 512 + 3 * 512], msg[64 + 512:64 + 512 + 3 * 512])
    # one hop: bf16(widen(in) + local), by torch's arithmetic
    msg2 = orc.dar_hop(ch, 1, msg, y)
    s = torch.from_numpy(want.view(np.int16)).view(torch.bfloat16).float() + torch.from_numpy(y[4 * 256:])
    assert np.array_equal(msg2[64 + 512:64 + 512 + 3 * 512].view(np.uint16),
                          s.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    out = orc.decompress(ch, msg2, x)
    assert np.array_equal(out[4 * 256:], (s.to(torch.bfloat16).float() + torch.from_numpy(x[4 * 256:])).numpy())
    plain = orc.decompress(ch, msg2)
    assert np.array_equal(plain[4 * 256:], s.to(torch.bfloat16).float().numpy())
    # the coded super-groups in front are what they would be without the 16-bit run
    ch3 = O.make_chunk(7, [1, 2, 1])
    assert np.array_equal(orc.compress(ch3, 0, x[:4 * 256])[:64 + 256 + 256], msg[:64 + 256 + 256])
    assert np.array_equal(orc.decompress(ch3, orc.compress(ch3, 0, x[:4 * 256])), orc.decompress(ch, msg)[:4 * 256])


def test_ring_with_sixteen_bit_run_is_exact_on_bf16_friendly_values():
    n = 4
    orc = O.Oracle(n, seed=2)
    rng = np.random.default_rng(6)
    counts = [0, 0, 0, 8]                                            # everything uncompressed
    gs = [(rng.integers(-8, 8, 8 * 256) * 2.0 ** -4).astype(np.float32) for _ in range(n)]   # sums stay exact in bf16
    out = np.concatenate(O.ring_reduce_scatter(orc, gs, counts))
    assert np.array_equal(out, sum(gs))
    out = np.concatenate(O.butterfly_reduce_scatter(orc, gs, counts))
    assert np.array_equal(out, sum(gs))


# ----------------------------------------------------------------- the permutation and long rings

def test_ring_error_grows_about_linearly_with_the_hops():
    """8-bit super-groups on rings of 16 and 64 workers: four times the hops, about four times
    the error.  (With neighbouring workers in neighbouring intervals -- a cyclic shift as the
    permutation -- the same pair of rings gives a ratio near 15 and 5 times the error at 64;
    tests/test_oracle_rounding_bias.py compares the law with an ideal shuffle.)"""
    def run(n):
        rng = np.random.default_rng(7)
        J = n
        gs = [(rng.standard_normal(J * 256) * 1e-3).astype(np.float32) for _ in range(n)]
        out = O.ring_reduce_scatter(O.Oracle(n, seed=11), gs, [0, 0, J])
        return vnmse(out, gs)
    e16, e64 = run(16), run(64)
    assert e64 < 2.5e-3 and 2.0 < e64 / e16 < 7.0, (e16, e64)


# ----------------------------------------------------------------- mean subtraction (Section 3.1)

@pytest.mark.parametrize("n", [2, 4, 8])
def test_schedules_subtract_each_workers_mean_exactly_once(n):
    """bf16 gradients and a mean per super-group: both schedules return bit for bit what they
    return on fp32 gradients from which the mean was taken off beforehand.  A mean subtracted
    twice (from a butterfly's fp32 buffer) or never (at one kind of node) would show."""
    J = 2 * n
    counts = [n // 2, n // 2, n - 2, 2]
    orc = O.Oracle(n, seed=17)
    gs = grads(n, J, 21, np.uint16)
    rng = np.random.default_rng(22)
    mu = (rng.standard_normal(J) * 3e-4).astype(np.float32)
    pre = [widen(g) - np.repeat(mu, 256) for g in gs]
    for fn in (O.ring_reduce_scatter, O.butterfly_reduce_scatter):
        got = np.concatenate(fn(orc, gs, counts, first_sg=5, mu=mu))
        want = np.concatenate(fn(orc, pre, counts, first_sg=5))
        assert np.array_equal(got, want), fn.__name__
        assert not np.array_equal(got, np.concatenate(fn(orc, gs, counts, first_sg=5)))


def test_mean_subtraction_removes_a_common_offset_from_the_error():
    """Entries c + noise: without the mean the 4-bit error is relative to c, with it to the noise."""
    n, J = 4, 8
    rng = np.random.default_rng(23)
    gs = [(1.0 + rng.standard_normal(J * 256) * 1e-2).astype(np.float32) for _ in range(n)]
    mu = np.mean([g.reshape(J, 256).mean(axis=1) for g in gs], axis=0).astype(np.float32)
    orc = O.Oracle(n, seed=4)
    truth = sum(g.astype(np.float64) for g in gs)
    plain = np.concatenate(O.ring_reduce_scatter(orc, gs, [0, J, 0])).astype(np.float64)
    normd = np.concatenate(O.ring_reduce_scatter(orc, gs, [0, J, 0], mu=mu)).astype(np.float64) + n * np.repeat(mu, 256).astype(np.float64)
    e_plain = ((plain - truth) ** 2).sum()
    e_normd = ((normd - truth) ** 2).sum()
    assert e_normd < e_plain / 100
