"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Bar: packed codes, u8 group scales, bf16 super-group scales and E8M0 bytes bit-exact;
fp32 decoded sums within 1e-6 relative (they are expected to be bit-exact too, the slack is
the tolerance the benchmark spec states for floating point).
"""
import numpy as np
import pytest
import torch

from oracle import dq_oracle as O
from paper_2602_08923_amd import binding as B
from paper_2602_08923_amd import prep, workloads

pytestmark = pytest.mark.gpu

RTOL = 1e-6


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


def to_dev(a, dev):
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    return torch.from_numpy(a).to(dev)


def host(t):
    return t.detach().cpu().numpy()


def make_local(rng, n, dtype, scale=1e-3):
    x = (rng.standard_normal(n) * scale).astype(np.float32)
    if dtype == "bf16":
        return (x.view(np.uint32) >> 16).astype(np.uint16)
    return x


def assert_close_f32(got, want):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    tol = RTOL * np.maximum(np.abs(want), np.abs(got)) + 1e-30
    bad = np.abs(got - want) > tol
    assert not bad.any(), f"{bad.sum()} of {bad.size} entries differ, first at {np.argmax(bad)}"


CASES = [
    # n_workers, n_sg (2,4,8 bit), first_sg, rank
    (4, [5, 7, 3], 0, 1),
    (8, [0, 9, 0], 2 ** 33 + 11, 7),
    (3, [1, 0, 2], 12345, 2),        # worker count that is not a power of two
    (64, [13, 0, 0], 7, 63),
    (1, [0, 1, 1], 0, 0),
    (100, [2, 66, 5], 999, 42),
    (6, [3, 3, 3], 5, 5),            # not a power of two: the permutation walks 3-bit integers until one is below 6
    (8192, [2, 4, 1], 2 ** 40, 8191),  # the largest worker count
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", CASES)
def test_single_chunk_calls_match_oracle(dev, dtype, case):
    n, n_sg, first_sg, rank = case
    seed, rnd = 0xC0FFEE1234, 5
    rng = np.random.default_rng(n * 1000 + sum(n_sg))
    entries = sum(n_sg) * 256
    orc = O.Oracle(n, seed=seed, round=rnd)
    ctx = B.Context(n, seed=seed, round=rnd)
    och, gch = O.make_chunk(first_sg, n_sg), B.make_chunk(first_sg, n_sg)
    assert B.dq_packed_bytes(gch) == O.Oracle.packed_bytes(och)

    a = make_local(rng, entries, dtype)
    b = make_local(rng, entries, dtype)
    c = make_local(rng, entries, dtype)
    # leaf
    want1 = orc.compress(och, rank, a)
    got1 = ctx.dq_compress(to_dev(a, dev), gch, rank)
    assert np.array_equal(host(got1), want1)
    # internal node (a different worker re-encodes)
    rank2 = (rank + 1) % n
    want2 = orc.dar_hop(och, rank2, want1, b)
    got2 = ctx.dq_dar_hop(got1, to_dev(b, dev), gch, rank2)
    assert np.array_equal(host(got2), want2)
    # in place
    got2b = got1.clone()
    ctx.dq_dar_hop(got2b, to_dev(b, dev), gch, rank2, packed_out=got2b)
    assert np.array_equal(host(got2b), want2)
    # sink, and plain decompress
    assert_close_f32(host(ctx.dq_decompress(got2, gch, local=to_dev(c, dev))), orc.decompress(och, want2, c))
    assert_close_f32(host(ctx.dq_decompress(got2, gch)), orc.decompress(och, want2))
    assert np.array_equal(host(ctx.dq_decompress(got2, gch)), orc.decompress(och, want2))
    ctx.close()


def test_new_round_draws_new_numbers(dev):
    n_sg = [1, 2, 1]
    rng = np.random.default_rng(4)
    a = make_local(rng, 4 * 256, "f32")
    ctx = B.Context(4, seed=9, round=0)
    gch = B.make_chunk(0, n_sg)
    p0 = host(ctx.dq_compress(to_dev(a, dev), gch, 0))
    ctx.set_round(1)
    p1 = host(ctx.dq_compress(to_dev(a, dev), gch, 0))
    assert not np.array_equal(p0, p1)
    assert np.array_equal(p1, O.Oracle(4, seed=9, round=1).compress(O.make_chunk(0, n_sg), 0, a))


def test_degenerate_inputs(dev):
    """All-zero chunk, signed zeros, values below the flush threshold, denormal groups,
    one huge outlier, exact powers of two, magnitudes whose reciprocal is denormal (there the
    normalised maximum can exceed 1 by an ulp before the rule's clamp)."""
    n, n_sg = 4, [2, 2, 2]
    entries = 6 * 256
    rng = np.random.default_rng(31)
    orc, ctx = O.Oracle(n, seed=1), B.Context(n, seed=1)
    och, gch = O.make_chunk(3, n_sg), B.make_chunk(3, n_sg)
    variants = []
    z = np.zeros(entries, np.float32)
    variants.append(z)
    s = z.copy(); s[::3] = -0.0
    variants.append(s)
    variants.append(np.full(entries, 2.0 ** -110, np.float32))
    d = (rng.standard_normal(entries) * 1e-3).astype(np.float32); d[16:48] = 1e-42; d[300:316] = 0.0
    variants.append(d)
    o = (rng.standard_normal(entries) * 1e-3).astype(np.float32); o[700] = 3.0e4
    variants.append(o)
    p = np.ldexp(1.0, rng.integers(-20, 3, entries)).astype(np.float32) * rng.choice([-1.0, 1.0], entries).astype(np.float32)
    variants.append(p)
    h = (rng.standard_normal(entries) * 2e37).astype(np.float32)
    big = np.array([0x7F4006EE], np.uint32).view(np.float32)[0]   # 2.55e38: big * fp32(1/big) = 1 + 2^-22
    assert np.float32(big * (np.float32(1.0) / big)) > 1.0
    h[5::256] = 1.5e38; h[6::256] = -1.5e38; h[40::256] = big; h[41::256] = -big; h[100::256] = big
    variants.append(h)
    prev_o = prev_g = None
    for v in variants:
        w = orc.compress(och, 2, v)
        g = ctx.dq_compress(to_dev(v, dev), gch, 2)
        assert np.array_equal(host(g), w)
        if prev_o is not None:
            w2 = orc.dar_hop(och, 3, prev_o, v)
            g2 = ctx.dq_dar_hop(prev_g, to_dev(v, dev), gch, 3)
            assert np.array_equal(host(g2), w2)
            assert np.array_equal(host(ctx.dq_decompress(g2, gch, local=to_dev(v, dev))), orc.decompress(och, w2, v))
        prev_o, prev_g = w, g


def test_empty_chunk_and_bad_arguments(dev):
    ctx = B.Context(4)
    empty = B.make_chunk(0, [0, 0, 0])
    assert B.dq_packed_bytes(empty) == 0
    buf = torch.zeros(16, dtype=torch.uint8, device=dev)
    loc = torch.zeros(0, dtype=torch.float32, device=dev)
    ctx.dq_compress(loc, empty, 0, packed_out=buf)  # nothing to do, no launch
    torch.cuda.synchronize()
    assert int(buf.sum()) == 0
    ch = B.make_chunk(0, [0, 1, 0])
    x = torch.zeros(256, dtype=torch.float32, device=dev)
    with pytest.raises(B.DqError):  # rank outside 0..n-1
        ctx.dq_compress(x, ch, 4)
    with pytest.raises(B.DqError):  # misaligned local
        ctx.dq_compress(torch.zeros(257, dtype=torch.float32, device=dev)[1:], ch, 0)
    with pytest.raises(B.DqError):
        B.Context(0)
    with pytest.raises(B.DqError):
        B.Context(4, g4=1.0)
    with pytest.raises(B.DqError):  # 8-bit level set too fine for the search table
        B.Context(4, g8=1.1)


@pytest.mark.parametrize("g4,g8", [(2.0, 1.04), (1.05, 1.005)])
def test_other_level_sets(dev, g4, g8):
    n, n_sg = 8, [0, 6, 6]
    rng = np.random.default_rng(77)
    a, b = make_local(rng, 12 * 256, "bf16"), make_local(rng, 12 * 256, "bf16")
    orc, ctx = O.Oracle(n, seed=3, g4=g4, g8=g8), B.Context(n, seed=3, g4=g4, g8=g8)
    och, gch = O.make_chunk(50, n_sg), B.make_chunk(50, n_sg)
    w1 = orc.compress(och, 0, a)
    g1 = ctx.dq_compress(to_dev(a, dev), gch, 0)
    assert np.array_equal(host(g1), w1)
    assert np.array_equal(host(ctx.dq_dar_hop(g1, to_dev(b, dev), gch, 5)), orc.dar_hop(och, 5, w1, b))


# ----------------------------------------------------------------------------- hop replay

def prepared(wl, dev, entries=None, bucket=0):
    """Worker gradients of one bucket on the device, reordered by the allocation."""
    grads = [workloads.draw(wl, w, bucket, device="cpu", entries=entries) for w in range(wl.n_workers)]
    re, counts, _ = prep.prepare_bucket(grads, wl.budget_bits, wl.n_workers)
    return re, counts


def test_ring_replay_config1_full(dev):
    """Benchmark configuration 1 at full size: 4 workers, 2^20 fp32 entries each, b = 5."""
    wl = workloads.CONFIGS[1]
    re, counts = prepared(wl, dev)
    assert sum(counts) == 4096 and counts[1] > 0
    orc, ctx = O.Oracle(4, seed=11), B.Context(4, seed=11)
    want = np.concatenate(O.ring_reduce_scatter(orc, [workloads.to_numpy(g) for g in re], counts))
    rp = B.Replay(ctx, B.DQ_RING, B.DQ_DYNAMIQ, [g.to(dev) for g in re], 4096, [counts])
    assert rp.n_steps == 4
    rp.run()
    torch.cuda.synchronize()
    got = host(rp.out)
    assert_close_f32(got, want)
    assert np.array_equal(got, want)
    # the sum is approximated, not garbage
    true = sum(g.double() for g in re).numpy()
    assert ((got - true) ** 2).sum() / (true ** 2).sum() < 0.05
    # replays are deterministic
    rp.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out), want)


def test_replay_launch_by_launch_equals_the_whole_replay(dev):
    """dq_replay_run_launch: every launch of every step, in order, is the replay (a butterfly step in
    which nodes forward and keep is two launches); a launch a step does not have is refused."""
    n, n_sg, counts = 8, 48, [[10, 30, 8]]
    rng = np.random.default_rng(77)
    grads = [to_dev(make_local(rng, n_sg * 256, "bf16"), dev) for _ in range(n)]
    ctx = B.Context(n, seed=9)
    rp = B.Replay(ctx, B.DQ_BUTTERFLY, B.DQ_DYNAMIQ, grads, n_sg, counts)
    rp.run()
    torch.cuda.synchronize()
    want = host(rp.out).copy()
    rp.out.zero_()
    kinds = [rp.step_info(t)[0] for t in range(rp.n_steps)]
    assert 3 in kinds                                   # some step both forwards and keeps
    for t, kind in enumerate(kinds):
        rp.run_launch(t, 0)
        if kind == 3:
            rp.run_launch(t, 1)
        else:
            with pytest.raises(B.DqError):
                rp.run_launch(t, 1)
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out), want)


def test_stream_probe_reads_and_writes_every_word(dev):
    """The measurement aid: out word j = xor of in words j, j + n_out, j + 2 n_out, ... (16-byte words)."""
    ctx = B.Context(4, seed=1)
    rng = np.random.default_rng(5)
    for n_in, n_out in ((64, 64), (1000, 64), (4096 + 3, 1024), (130, 129)):
        src = rng.integers(0, 2 ** 32, size=(n_in, 4), dtype=np.uint32)
        want = np.zeros((n_out, 4), np.uint32)
        for j in range(n_out):
            want[j] = np.bitwise_xor.reduce(src[j::n_out], axis=0)
        s = torch.from_numpy(src.view(np.uint8).reshape(-1).copy()).to(dev)
        d = torch.full((n_out * 16,), 0xEE, dtype=torch.uint8, device=dev)
        B.dq_stream_probe(ctx, s, d)
        torch.cuda.synchronize()
        assert np.array_equal(host(d).view(np.uint32).reshape(n_out, 4), want), (n_in, n_out)


@pytest.mark.parametrize("topology", ["ring", "butterfly"])
def test_replay_captured_in_a_graph(dev, topology):
    """A replay is kernel launches only (no memset, no copy, no event), so a caller may capture it in
    a HIP graph.  The graph is replayed three times, with eager work of the program and
    synchronisations between the replays (the gradients change in place); every replay must equal the
    eager replay on the same inputs, and the first the oracle."""
    n, n_sg, counts = 8, 64, [[20, 36, 8]]
    rng = np.random.default_rng(31)
    grads = [make_local(rng, n_sg * 256, "bf16") for _ in range(n)]
    dev_grads = [to_dev(g, dev) for g in grads]
    topo = B.DQ_RING if topology == "ring" else B.DQ_BUTTERFLY
    orc, ctx = O.Oracle(n, seed=41), B.Context(n, seed=41)
    reduce = O.ring_reduce_scatter if topology == "ring" else O.butterfly_reduce_scatter
    want = np.concatenate(reduce(orc, grads, counts[0]))
    rp = B.Replay(ctx, topo, B.DQ_DYNAMIQ, dev_grads, n_sg, counts)
    rp.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out), want)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        rp.run()                                   # warm-up on the capturing stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            rp.run()
    torch.cuda.synchronize()
    for k in range(3):
        for g in dev_grads:                        # eager work between the replays
            g.mul_(-1.25 - k)
        torch.cuda.synchronize()
        rp.out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = host(rp.out).copy()
        rp.out.zero_()
        rp.run()
        torch.cuda.synchronize()
        assert np.array_equal(got, host(rp.out)), f"replay {k}"
        assert np.abs(got).max() > 0


@pytest.mark.parametrize("n,n_sg_bucket,counts,buckets", [(2, 8, [[2, 4, 2]], 1), (4, 12, [[3, 6, 3], [0, 12, 0]], 2),
                                                          (8, 40, [[7, 22, 11]], 1)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_butterfly_replay_small(dev, n, n_sg_bucket, counts, buckets, dtype):
    rng = np.random.default_rng(n + buckets)
    d = n_sg_bucket * 256
    grads = [make_local(rng, d * buckets, dtype) for _ in range(n)]
    orc, ctx = O.Oracle(n, seed=21, round=1), B.Context(n, seed=21, round=1)
    want = []
    for b in range(buckets):
        want += O.butterfly_reduce_scatter(orc, [g[b * d:(b + 1) * d] for g in grads], counts[b],
                                           first_sg=100 + b * n_sg_bucket)
    want = np.concatenate(want)
    rp = B.Replay(ctx, B.DQ_BUTTERFLY, B.DQ_DYNAMIQ, [to_dev(g, dev) for g in grads], n_sg_bucket, counts,
                  n_buckets=buckets, first_sg=100)
    rp.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out), want)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ring_and_chain_replay_small(dev, dtype):
    n, n_sg_bucket, counts = 4, 20, [[4, 11, 5], [20, 0, 0]]
    rng = np.random.default_rng(5)
    d = n_sg_bucket * 256
    grads = [make_local(rng, 2 * d, dtype) for _ in range(n)]
    orc, ctx = O.Oracle(n, seed=2), B.Context(n, seed=2)
    want = []
    for b in range(2):
        want += O.ring_reduce_scatter(orc, [g[b * d:(b + 1) * d] for g in grads], counts[b], first_sg=b * n_sg_bucket)
    rp = B.Replay(ctx, B.DQ_RING, B.DQ_DYNAMIQ, [to_dev(g, dev) for g in grads], n_sg_bucket, counts, n_buckets=2)
    ms = rp.run(timed=True)
    assert len(ms) == 4 and all(m >= 0 for m in ms)
    assert [rp.step_info(i)[0] for i in range(4)] == [0, 1, 1, 2]
    assert rp.step_info(1)[1] == 2 * d
    assert np.array_equal(host(rp.out), np.concatenate(want))
    # chain: the path of one chunk through all n workers
    och = O.make_chunk(77, [3, 5, 2])
    sl = [make_local(rng, 2560, dtype) for _ in range(n)]
    msg = orc.compress(och, 0, sl[0])
    for i in (1, 2):
        msg = orc.dar_hop(och, i, msg, sl[i])
    want = orc.decompress(och, msg, sl[3])
    rc = B.Replay(ctx, B.DQ_CHAIN, B.DQ_DYNAMIQ, [to_dev(s, dev) for s in sl], 10, [[3, 5, 2]], first_sg=77)
    rc.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rc.out), want)


# ----------------------------------------------------------------------------- MX codec

@pytest.mark.parametrize("fmt", [B.DQ_MXFP8_E4M3, B.DQ_MXFP6_E3M2, B.DQ_MXFP4_E2M1])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_mx_calls_match_oracle(dev, fmt, dtype):
    rng = np.random.default_rng(fmt)
    n = 256 * 37
    a = make_local(rng, n, dtype)
    b = make_local(rng, n, dtype, scale=3e-3)
    if dtype == "f32":
        a[100:132] = 0.0           # an all-zero block
        a[200] = 1e-41             # denormal
        a[300] = 448.0 * 2.0 ** -3  # a block maximum exactly on a power-of-two boundary case
        a[5000] = 3.0e38           # near the top of binary32
    assert B.dq_mx_packed_bytes(fmt, n) == O.mx_packed_bytes(fmt, n)
    w1 = O.mx_compress(fmt, a)
    g1 = B.dq_mx_compress(fmt, to_dev(a, dev))
    assert np.array_equal(host(g1), w1)
    w2 = O.mx_dar_hop(fmt, w1, b)
    g2 = B.dq_mx_dar_hop(fmt, g1, to_dev(b, dev))
    assert np.array_equal(host(g2), w2)
    assert np.array_equal(host(B.dq_mx_decompress(fmt, g2, n)), O.mx_decompress(fmt, w2, n))
    assert np.array_equal(host(B.dq_mx_decompress(fmt, g2, n, local=to_dev(a, dev))), O.mx_decompress(fmt, w2, n, a))


@pytest.mark.parametrize("fmt", [B.DQ_MXFP8_E4M3, B.DQ_MXFP6_E3M2, B.DQ_MXFP4_E2M1])
def test_mx_every_code_roundtrips(dev, fmt):
    """decode(encode) is the identity on every element code at several block scales."""
    bits = O.MX_CODE_BITS[fmt]
    codes = [c for c in range(1 << bits) if not (fmt == B.DQ_MXFP8_E4M3 and (c & 0x7F) == 0x7F)]
    for e in (1, 100, 127, 200):
        vals = np.array([O.mx_decode_elem(fmt, c, e) for c in codes], np.float32)
        blocks = []
        top = max(abs(float(v)) for v in vals)
        # pad every block with the format's largest value so that the shared exponent is e
        for i in range(0, len(vals), 31):
            blk = np.full(32, top, np.float32)
            part = vals[i:i + 31]
            blk[1:1 + len(part)] = part
            blocks.append(blk)
        x = np.concatenate(blocks)
        x = np.concatenate([x, np.zeros((-len(x)) % 256, np.float32)])
        g = B.dq_mx_compress(fmt, to_dev(x, dev))
        assert np.array_equal(host(g), O.mx_compress(fmt, x))
        back = host(B.dq_mx_decompress(fmt, g, len(x)))
        assert np.array_equal(back, x)


def test_mx_ring_replay_small(dev):
    n = 4
    rng = np.random.default_rng(12)
    grads = [make_local(rng, 16 * 256, "bf16") for _ in range(n)]
    ctx = B.Context(n)
    for fmt in (B.DQ_MXFP8_E4M3, B.DQ_MXFP6_E3M2, B.DQ_MXFP4_E2M1):
        want = np.concatenate(O.mx_ring_reduce_scatter(fmt, grads))
        rp = B.Replay(ctx, B.DQ_RING, fmt, [to_dev(g, dev) for g in grads], 16)
        rp.run()
        torch.cuda.synchronize()
        assert np.array_equal(host(rp.out), want)


# ----------------------------------------------------------------------------- launch shape

def test_result_does_not_depend_on_launch_shape(dev, monkeypatch):
    """The same chunk under different grid sizes, and cut in two calls, gives the same bytes:
    the random streams are keyed by global indices, not by the grid."""
    n, n_sg = 8, [3700, 15000, 2100]
    rng = np.random.default_rng(99)
    entries = sum(n_sg) * 256
    a, b = make_local(rng, entries, "bf16"), make_local(rng, entries, "bf16")
    orc = O.Oracle(n, seed=5)
    och, gch = O.make_chunk(4000, n_sg), B.make_chunk(4000, n_sg)
    want1 = orc.compress(och, 2, a)
    want2 = orc.dar_hop(och, 3, want1, b)
    want3 = orc.decompress(och, want2, a)
    monkeypatch.delenv("DQ_BLOCKS_PER_CU", raising=False)
    for per_cu in ("1", "2", "7", "64"):   # from ~7 tiles per wave down to one
        monkeypatch.setenv("DQ_BLOCKS_PER_CU", per_cu)
        ctx = B.Context(n, seed=5)
        g1 = ctx.dq_compress(to_dev(a, dev), gch, 2)
        g2 = ctx.dq_dar_hop(g1, to_dev(b, dev), gch, 3)
        assert np.array_equal(host(g1), want1) and np.array_equal(host(g2), want2)
        assert np.array_equal(host(ctx.dq_decompress(g2, gch, local=to_dev(a, dev))), want3)
    # split the 4-bit run in two chunks: codes of the second part must match the tail of the whole
    ctx = B.Context(n, seed=5)
    monkeypatch.delenv("DQ_BLOCKS_PER_CU", raising=False)
    n_a, n_b = [3700, 7000, 0], [0, 8000, 2100]
    ea = sum(n_a) * 256
    ga = ctx.dq_compress(to_dev(a[:ea], dev), B.make_chunk(4000, n_a), 2)
    gb = ctx.dq_compress(to_dev(a[ea:], dev), B.make_chunk(4000 + sum(n_a), n_b), 2)
    wa = orc.compress(O.make_chunk(4000, n_a), 2, a[:ea])
    wb = orc.compress(O.make_chunk(4000 + sum(n_a), n_b), 2, a[ea:])
    assert np.array_equal(host(ga), wa) and np.array_equal(host(gb), wb)
    whole = want1
    assert np.array_equal(wa[:3700 * 64], whole[:3700 * 64])                       # 2-bit codes
    assert np.array_equal(wa[3700 * 64:3700 * 64 + 7000 * 128], whole[3700 * 64:3700 * 64 + 7000 * 128])  # first 4-bit codes
    assert np.array_equal(wb[:8000 * 128], whole[3700 * 64 + 7000 * 128:3700 * 64 + 15000 * 128])         # the other 4-bit codes


# ----------------------------------------------------------------------------- all-gather phase

@pytest.mark.parametrize("topology", ["ring", "butterfly"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_all_gather_phase(dev, topology, dtype):
    """Reduce-scatter followed by the all-gather: every worker ends with decompress(compress(sum))."""
    n, n_sg = 8, 8 * 9
    rng = np.random.default_rng(31)
    grads = [make_local(rng, n_sg * 256, dtype) for _ in range(n)]
    counts = [20, 41, 11]
    orc = O.Oracle(n, seed=5)
    rs = (O.ring_reduce_scatter if topology == "ring" else O.butterfly_reduce_scatter)(orc, grads, counts, first_sg=1000)
    want = np.concatenate(O.all_gather(orc, rs, counts, topology, first_sg=1000))
    ctx = B.Context(n, seed=5)
    topo = B.DQ_RING if topology == "ring" else B.DQ_BUTTERFLY
    rp = B.Replay(ctx, topo, B.DQ_DYNAMIQ, [to_dev(g, dev) for g in grads], n_sg, [counts], first_sg=1000, all_gather=True)
    base = B.Replay(ctx, topo, B.DQ_DYNAMIQ, [to_dev(g, dev) for g in grads], n_sg, [counts], first_sg=1000)
    assert rp.n_steps == base.n_steps + 2
    assert [rp.step_info(i)[0] for i in (rp.n_steps - 2, rp.n_steps - 1)] == [0, 2]
    rp.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out), want)
    # the result is not the reduce-scatter's: one more quantization happened
    assert not np.array_equal(want, np.concatenate(rs))


def test_all_gather_phase_mx_and_chain(dev):
    n, n_sg = 4, 4 * 6
    rng = np.random.default_rng(32)
    grads = [make_local(rng, n_sg * 256, "bf16") for _ in range(n)]
    rs = O.mx_ring_reduce_scatter(B.DQ_MXFP6_E3M2, grads)
    want = np.concatenate(O.mx_all_gather(B.DQ_MXFP6_E3M2, rs))
    ctx = B.Context(n)
    rp = B.Replay(ctx, B.DQ_RING, B.DQ_MXFP6_E3M2, [to_dev(g, dev) for g in grads], n_sg, all_gather=True)
    rp.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out), want)
    # chain: one chunk, the last worker is the sink
    counts = [5, 12, 7]
    orc = O.Oracle(n, seed=9)
    ch = O.make_chunk(0, counts)
    msg = orc.compress(ch, 0, grads[0])
    for i in range(1, n - 1):
        msg = orc.dar_hop(ch, i, msg, grads[i])
    total = orc.decompress(ch, msg, grads[n - 1])
    want = orc.decompress(ch, orc.compress(ch, n - 1, total))
    rc = B.Replay(B.Context(n, seed=9), B.DQ_CHAIN, B.DQ_DYNAMIQ, [to_dev(g, dev) for g in grads], n_sg, [counts], all_gather=True)
    rc.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rc.out), want)


# ----------------------------------------------------------------------------- 16-bit (uncompressed) super-groups

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_sg", [[3, 5, 2, 7], [0, 0, 0, 9], [1, 0, 0, 1], [0, 6, 0, 130], [5, 5, 5, 0]])
def test_sixteen_bit_run(dev, dtype, n_sg):
    """Chunks with a run of raw-bf16 super-groups behind the coded ones: every call against the oracle."""
    n = 4
    total = sum(n_sg) * 256
    rng = np.random.default_rng(sum(n_sg))
    a = make_local(rng, total, dtype)
    b = make_local(rng, total, dtype, scale=3e-3)
    orc = O.Oracle(n, seed=3)
    och, gch = O.make_chunk(500, n_sg), B.make_chunk(500, n_sg)
    assert B.dq_packed_bytes(gch) == O.Oracle.packed_bytes(och)
    ctx = B.Context(n, seed=3)
    w1 = orc.compress(och, 1, a)
    g1 = ctx.dq_compress(to_dev(a, dev), gch, 1)
    assert np.array_equal(host(g1), w1)
    w2 = orc.dar_hop(och, 2, w1, b)
    g2 = ctx.dq_dar_hop(g1, to_dev(b, dev), gch, 2)
    assert np.array_equal(host(g2), w2)
    assert np.array_equal(host(ctx.dq_decompress(g2, gch)), orc.decompress(och, w2))
    assert np.array_equal(host(ctx.dq_decompress(g2, gch, local=to_dev(a, dev))), orc.decompress(och, w2, a))


@pytest.mark.parametrize("topology", ["ring", "butterfly"])
def test_replay_with_sixteen_bit_run(dev, topology):
    n, n_sg = 8, 8 * 11
    rng = np.random.default_rng(41)
    grads = [make_local(rng, n_sg * 256, "bf16") for _ in range(n)]
    counts = [13, 30, 22, 23]
    orc = O.Oracle(n, seed=6)
    rs = (O.ring_reduce_scatter if topology == "ring" else O.butterfly_reduce_scatter)(orc, grads, counts, first_sg=64)
    want = np.concatenate(O.all_gather(orc, rs, counts, topology, first_sg=64))
    ctx = B.Context(n, seed=6)
    topo = B.DQ_RING if topology == "ring" else B.DQ_BUTTERFLY
    rp = B.Replay(ctx, topo, B.DQ_DYNAMIQ, [to_dev(g, dev) for g in grads], n_sg, [counts], first_sg=64, all_gather=True)
    rp.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out), want)


def test_more_jobs_than_grid_rows(dev):
    """512-worker recursive halving: the first steps have 131,072 and 65,536 (worker, chunk) jobs,
    more than one launch's 65,535 grid rows, so they are split over launches."""
    n = 512
    n_sg = n
    rng = np.random.default_rng(77)
    grads = [make_local(rng, n_sg * 256, "bf16") for _ in range(n)]
    counts = [100, 300, 112]
    want = np.concatenate(O.butterfly_reduce_scatter(O.Oracle(n, seed=4), grads, counts))
    ctx = B.Context(n, seed=4)
    rp = B.Replay(ctx, B.DQ_BUTTERFLY, B.DQ_DYNAMIQ, [to_dev(g, dev) for g in grads], n_sg, [counts])
    rp.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out), want)
    rm = B.Replay(ctx, B.DQ_BUTTERFLY, B.DQ_MXFP4_E2M1, [to_dev(g, dev) for g in grads], n_sg)
    rm.run()
    torch.cuda.synchronize()
    true = sum((g.astype(np.uint32) << 16).view(np.float32).astype(np.float64) for g in grads)
    got = host(rm.out).astype(np.float64)
    assert ((got - true) ** 2).sum() / (true ** 2).sum() < 0.2


def test_independent_rounding_mode(dev):
    """dq_config.independent_rounding: u = gamma for every worker (the baseline of Section 2.4)."""
    n, n_sg = 8, [9, 14, 9]
    total = sum(n_sg) * 256
    rng = np.random.default_rng(8)
    a, b = make_local(rng, total, "bf16"), make_local(rng, total, "bf16")
    orc = O.Oracle(n, seed=2, independent=True)
    och, gch = O.make_chunk(10, n_sg), B.make_chunk(10, n_sg)
    ctx = B.Context(n, seed=2, independent_rounding=True)
    w1 = orc.compress(och, 3, a)
    g1 = ctx.dq_compress(to_dev(a, dev), gch, 3)
    assert np.array_equal(host(g1), w1)
    assert np.array_equal(host(ctx.dq_dar_hop(g1, to_dev(b, dev), gch, 5)), orc.dar_hop(och, 5, w1, b))
    assert not np.array_equal(w1, O.Oracle(n, seed=2).compress(och, 3, a))      # not the correlated codes
    grads = [make_local(rng, 32 * 256, "bf16") for _ in range(n)]
    want = np.concatenate(O.ring_reduce_scatter(orc, grads, [8, 16, 8]))
    rp = B.Replay(ctx, B.DQ_RING, B.DQ_DYNAMIQ, [to_dev(g, dev) for g in grads], 32, [[8, 16, 8]])
    rp.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out), want)


# ----------------------------------------------------------------------------- block-wise pipelining

def block_chunks(n_sg, block_sg, first_sg):
    counts = list(n_sg) + [0] * (4 - len(n_sg))
    edges = np.cumsum([0] + counts)
    total = int(edges[-1])
    out = []
    for lo in range(0, total, block_sg):
        hi = min(lo + block_sg, total)
        out.append((lo, hi, [int(max(0, min(hi, edges[w + 1]) - max(lo, edges[w]))) for w in range(4)]))
    return [(lo, hi, O.make_chunk(first_sg + lo, c)) for lo, hi, c in out]


@pytest.mark.parametrize("block_sg", [4, 7, 64, 1000])
def test_pipelined_hops_match_blockwise_oracle(dev, block_sg):
    """Section 4: a chunk travels in blocks, each a packed chunk of its own; three hops in a row."""
    n, n_sg, first = 4, [30, 41, 20, 9], 300
    total = sum(n_sg)
    rng = np.random.default_rng(block_sg)
    xs = [make_local(rng, total * 256, "bf16") for _ in range(3)]
    orc = O.Oracle(n, seed=12)
    ctx = B.Context(n, seed=12)
    gch = B.make_chunk(first, n_sg)
    blocks = block_chunks(n_sg, block_sg, first)
    want, msgs = [], [None] * len(blocks)
    for hop, x in enumerate(xs):
        for i, (lo, hi, ch) in enumerate(blocks):
            sl = x[lo * 256:hi * 256]
            msgs[i] = orc.compress(ch, hop, sl) if hop == 0 else orc.dar_hop(ch, hop, msgs[i], sl)
    for m in msgs:
        want.append(np.concatenate([m, np.zeros((-len(m)) % 256, np.uint8)]))
    want = np.concatenate(want)
    assert B.dq_pipelined_wire_bytes(gch, block_sg) == want.size
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    wire = None
    # a stage full of ones: a block's padding must reach the wire as zero all the same
    stage = torch.full((B.dq_pipelined_stage_bytes(gch, block_sg),), 0xFF, dtype=torch.uint8, device=dev)
    for hop, x in enumerate(xs):
        wire = B.dq_dar_hop_pipelined(ctx, wire, to_dev(x, dev), gch, hop, block_sg, s1, s2, stage=stage)
        s1.synchronize()
    assert np.array_equal(host(wire), want)
    with pytest.raises(B.DqError):
        B.dq_dar_hop_pipelined(ctx, wire, to_dev(xs[0], dev), gch, 0, block_sg, s1, s1)     # one stream: no overlap possible


# ----------------------------------------------------------------------------- mean subtraction (Section 3.1)

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_sg", [[5, 7, 3, 0], [1, 2, 1, 6], [0, 0, 13, 0], [9, 0, 0, 1]])
def test_single_chunk_calls_with_means(dev, dtype, n_sg):
    n, first, rank = 8, 1000, 3
    total = sum(n_sg)
    rng = np.random.default_rng(total)
    a, b, c = (make_local(rng, total * 256, dtype) for _ in range(3))
    mu = (rng.standard_normal(total) * 2e-4).astype(np.float32)
    mu_t = torch.from_numpy(mu).to(dev)
    orc, ctx = O.Oracle(n, seed=31, round=2), B.Context(n, seed=31, round=2)
    och, gch = O.make_chunk(first, n_sg), B.make_chunk(first, n_sg)
    w1 = orc.compress(och, rank, a, mu)
    g1 = ctx.dq_compress(to_dev(a, dev), gch, rank, mu=mu_t)
    assert np.array_equal(host(g1), w1)
    assert not np.array_equal(w1, orc.compress(och, rank, a))
    w2 = orc.dar_hop(och, rank + 1, w1, b, mu)
    g2 = ctx.dq_dar_hop(g1, to_dev(b, dev), gch, rank + 1, mu=mu_t)
    assert np.array_equal(host(g2), w2)
    assert np.array_equal(host(ctx.dq_decompress(g2, gch, local=to_dev(c, dev), mu=mu_t)), orc.decompress(och, w2, c, mu))
    assert np.array_equal(host(ctx.dq_decompress(g2, gch, mu=mu_t)), orc.decompress(och, w2))   # no local: means ignored
    with pytest.raises(B.DqError):
        ctx.dq_compress(to_dev(a, dev), gch, rank, mu=mu_t[:-1] if total > 1 else torch.zeros(2, device=dev))


@pytest.mark.parametrize("topology,n", [("ring", 4), ("ring", 5), ("butterfly", 2), ("butterfly", 4), ("butterfly", 16)])
def test_replay_with_means(dev, topology, n):
    """The means are taken off every worker's raw gradient exactly once, never off a butterfly's fp32 buffers."""
    J, buckets = 3 * n, 2
    counts = [[n, n // 2, n, 3 * n - 2 * n - n // 2], [0, 2 * n, n, 0]]
    rng = np.random.default_rng(n)
    d = J * 256
    grads = [make_local(rng, d * buckets, "bf16") for _ in range(n)]
    mu = (rng.standard_normal(J * buckets) * 2e-4).astype(np.float32)
    orc, ctx = O.Oracle(n, seed=9), B.Context(n, seed=9)
    fn = O.ring_reduce_scatter if topology == "ring" else O.butterfly_reduce_scatter
    want = []
    for b in range(buckets):
        rs = fn(orc, [g[b * d:(b + 1) * d] for g in grads], counts[b], first_sg=50 + b * J, mu=mu[b * J:(b + 1) * J])
        want += O.all_gather(orc, rs, counts[b], topology, first_sg=50 + b * J)
    topo = B.DQ_RING if topology == "ring" else B.DQ_BUTTERFLY
    rp = B.Replay(ctx, topo, B.DQ_DYNAMIQ, [to_dev(g, dev) for g in grads], J, counts, n_buckets=buckets, first_sg=50,
                  all_gather=True, mu=torch.from_numpy(mu).to(dev))
    rp.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out), np.concatenate(want))


def test_chain_and_pipelined_hops_with_means(dev):
    n, n_sg, first = 4, [6, 9, 4, 3], 40
    total = sum(n_sg)
    rng = np.random.default_rng(3)
    sl = [make_local(rng, total * 256, "bf16") for _ in range(n)]
    mu = (rng.standard_normal(total) * 2e-4).astype(np.float32)
    mu_t = torch.from_numpy(mu).to(dev)
    orc, ctx = O.Oracle(n, seed=14), B.Context(n, seed=14)
    och, gch = O.make_chunk(first, n_sg), B.make_chunk(first, n_sg)
    msg = orc.compress(och, 0, sl[0], mu)
    for i in (1, 2):
        msg = orc.dar_hop(och, i, msg, sl[i], mu)
    want = orc.decompress(och, msg, sl[3], mu)
    rc = B.Replay(ctx, B.DQ_CHAIN, B.DQ_DYNAMIQ, [to_dev(s, dev) for s in sl], total, [n_sg], first_sg=first, mu=mu_t)
    rc.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rc.out), want)
    # block-wise: block i takes the means of its own super-groups
    block_sg = 5
    blocks = block_chunks(n_sg, block_sg, first)
    msgs = [None] * len(blocks)
    for hop in range(2):
        for i, (lo, hi, ch) in enumerate(blocks):
            x = sl[hop][lo * 256:hi * 256]
            msgs[i] = orc.compress(ch, hop, x, mu[lo:hi]) if hop == 0 else orc.dar_hop(ch, hop, msgs[i], x, mu[lo:hi])
    want = np.concatenate([np.concatenate([m, np.zeros((-len(m)) % 256, np.uint8)]) for m in msgs])
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    wire = None
    for hop in range(2):
        wire = B.dq_dar_hop_pipelined(ctx, wire, to_dev(sl[hop], dev), gch, hop, block_sg, s1, s2, mu=mu_t)
        s1.synchronize()
    assert np.array_equal(host(wire), want)


def test_mx_replay_rejects_means(dev):
    n = 2
    grads = [torch.zeros(2 * 256, dtype=torch.float32, device=dev) for _ in range(n)]
    with pytest.raises(B.DqError):
        B.Replay(B.Context(n), B.DQ_RING, B.DQ_MXFP8_E4M3, grads, 2, mu=torch.zeros(2, device=dev))


# ----------------------------------------------------------------------------- restore fused into the last kernel

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_sg", [[5, 7, 3, 0], [1, 2, 1, 6], [0, 0, 1, 0], [9, 0, 4, 1]])
def test_decompress_restore_is_decompress_then_restore(dev, dtype, n_sg):
    from oracle import pp_oracle as P
    n, first = 8, 77
    total = sum(n_sg)
    rng = np.random.default_rng(total + 1)
    a, c = make_local(rng, total * 256, dtype), make_local(rng, total * 256, dtype)
    mu = (rng.standard_normal(total) * 2e-4).astype(np.float32)
    origin = rng.permutation(total).astype(np.uint32)          # reordered place p came from origin[p]
    pos = np.argsort(origin).astype(np.uint32)                 # pos[j] = place of original super-group j
    orc, ctx = O.Oracle(n, seed=3), B.Context(n, seed=3)
    och, gch = O.make_chunk(first, n_sg), B.make_chunk(first, n_sg)
    msg = orc.compress(och, 2, a, mu)
    msg_t = torch.from_numpy(msg).to(dev)
    mu_t, origin_t = torch.from_numpy(mu).to(dev), torch.from_numpy(origin.view(np.int32)).to(dev)
    for local, back in ((c, mu), (None, mu), (c, None), (None, None)):
        plain = orc.decompress(och, msg, local, mu if local is not None else None)
        want = P.restore(plain, pos, back, n)
        out = torch.full((total * 256,), float("nan"), dtype=torch.float32, device=dev)
        ctx.dq_decompress_restore(msg_t, gch, origin_t, out, local=None if local is None else to_dev(local, dev),
                                  mu=mu_t if local is not None else None, mu_back=None if back is None else mu_t)
        assert np.array_equal(host(out).view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("topology,n,all_gather", [("ring", 4, True), ("ring", 3, False), ("butterfly", 2, False),
                                                   ("butterfly", 8, True), ("butterfly", 4, False)])
def test_replay_writes_the_restored_result(dev, topology, n, all_gather):
    """dq_replay_desc.origin: the schedule's last launch scatters to the original order and adds n * mu."""
    from oracle import pp_oracle as P
    J, buckets = 4 * n, 2
    rng = np.random.default_rng(10 * n + all_gather)
    d = J * 256
    grads = [make_local(rng, d * buckets, "bf16") for _ in range(n)]     # already reordered
    widths = [np.sort(rng.choice(np.array([2, 4, 8, 16], np.uint8), J)) for _ in range(buckets)]
    counts = [[int((w == b).sum()) for b in (2, 4, 8, 16)] for w in widths]
    mu = (rng.standard_normal(J * buckets) * 2e-4).astype(np.float32)
    for b in range(buckets):
        mu[b * J + J - counts[b][3]:(b + 1) * J] = 0                      # 16-bit super-groups are not normalized
    origin = np.concatenate([rng.permutation(J) for _ in range(buckets)]).astype(np.uint32)
    orc, ctx = O.Oracle(n, seed=19), B.Context(n, seed=19)
    fn = O.ring_reduce_scatter if topology == "ring" else O.butterfly_reduce_scatter
    want = []
    for b in range(buckets):
        m = mu[b * J:(b + 1) * J]
        rs = fn(orc, [g[b * d:(b + 1) * d] for g in grads], counts[b], first_sg=b * J, mu=m)
        if all_gather:
            rs = O.all_gather(orc, rs, counts[b], topology, first_sg=b * J)
        pos = np.argsort(origin[b * J:(b + 1) * J]).astype(np.uint32)
        want.append(P.restore(np.concatenate(rs), pos, m, n))
    topo = B.DQ_RING if topology == "ring" else B.DQ_BUTTERFLY
    rp = B.Replay(ctx, topo, B.DQ_DYNAMIQ, [to_dev(g, dev) for g in grads], J, counts, n_buckets=buckets,
                  all_gather=all_gather, mu=torch.from_numpy(mu).to(dev),
                  origin=torch.from_numpy(origin.view(np.int32)).to(dev))
    rp.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out).view(np.uint32), np.concatenate(want).view(np.uint32))


# ----------------------------------------------------------------------------- reorder done by addressing

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_sg", [[5, 7, 3, 0], [1, 2, 1, 6], [0, 0, 1, 0], [9, 0, 4, 1]])
def test_gathered_local_equals_reordered_local(dev, dtype, n_sg):
    """dq_local.sg_index: the kernels read super-group j of the chunk at index sg_index[j] of the original tensor."""
    n, first = 8, 500
    total = sum(n_sg)
    extra = 5                                                   # the tensor is larger than the chunk
    rng = np.random.default_rng(total + 7)
    orig = [make_local(rng, (total + extra) * 256, dtype) for _ in range(3)]
    idx = rng.permutation(total + extra)[:total].astype(np.int32)
    mu = (rng.standard_normal(total) * 2e-4).astype(np.float32)

    def gathered(x):
        return np.ascontiguousarray(x.reshape(-1, 256)[idx].reshape(-1))

    idx_t, mu_t = torch.from_numpy(idx).to(dev), torch.from_numpy(mu).to(dev)
    orc, ctx = O.Oracle(n, seed=23), B.Context(n, seed=23)
    och, gch = O.make_chunk(first, n_sg), B.make_chunk(first, n_sg)
    w1 = orc.compress(och, 1, gathered(orig[0]), mu)
    g1 = ctx.dq_compress(to_dev(orig[0], dev), gch, 1, mu=mu_t, sg_index=idx_t)
    assert np.array_equal(host(g1), w1)
    w2 = orc.dar_hop(och, 2, w1, gathered(orig[1]), mu)
    g2 = ctx.dq_dar_hop(g1, to_dev(orig[1], dev), gch, 2, mu=mu_t, sg_index=idx_t)
    assert np.array_equal(host(g2), w2)
    want = orc.decompress(och, w2, gathered(orig[2]), mu)
    got = ctx.dq_decompress(g2, gch, local=to_dev(orig[2], dev), mu=mu_t, sg_index=idx_t)
    assert np.array_equal(host(got).view(np.uint32), want.view(np.uint32))
    with pytest.raises(B.DqError):
        ctx.dq_compress(to_dev(orig[0], dev), gch, 1, sg_index=idx_t + 10 ** 6)      # outside the tensor


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("topology,n,all_gather", [("ring", 4, True), ("ring", 3, False), ("butterfly", 2, False),
                                                   ("butterfly", 8, True), ("butterfly", 4, False)])
def test_replay_on_original_tensors(dev, topology, n, all_gather, dtype):
    """inputs_in_original_order: no reorder pass; gather on the way in, scatter and n * mu on the way out."""
    from oracle import pp_oracle as P
    J, buckets = 4 * n, 2
    rng = np.random.default_rng(100 * n + all_gather)
    d = J * 256
    orig = [make_local(rng, d * buckets, dtype) for _ in range(n)]
    widths = [rng.choice(np.array([2, 4, 8, 16], np.uint8), J) for _ in range(buckets)]
    pc = [P.positions(w) for w in widths]
    pos = np.concatenate([p for p, _ in pc])
    counts = [c for _, c in pc]
    mu = (rng.standard_normal(J * buckets) * 2e-4).astype(np.float32)
    mu_main = np.concatenate([P.reorder_mean(mu[b * J:(b + 1) * J], pos[b * J:(b + 1) * J], counts[b][3]) for b in range(buckets)])
    origin = np.concatenate([np.argsort(pos[b * J:(b + 1) * J]) for b in range(buckets)]).astype(np.int32)
    orc, ctx = O.Oracle(n, seed=29), B.Context(n, seed=29)
    fn = O.ring_reduce_scatter if topology == "ring" else O.butterfly_reduce_scatter
    want = []
    for b in range(buckets):
        pb = pos[b * J:(b + 1) * J]
        re = [P.reorder(g[b * d:(b + 1) * d], pb) for g in orig]
        rs = fn(orc, re, counts[b], first_sg=b * J, mu=mu_main[b * J:(b + 1) * J])
        if all_gather:
            rs = O.all_gather(orc, rs, counts[b], topology, first_sg=b * J)
        want.append(P.restore(np.concatenate(rs), pb, mu_main[b * J:(b + 1) * J], n))
    topo = B.DQ_RING if topology == "ring" else B.DQ_BUTTERFLY
    rp = B.Replay(ctx, topo, B.DQ_DYNAMIQ, [to_dev(g, dev) for g in orig], J, counts, n_buckets=buckets,
                  all_gather=all_gather, mu=torch.from_numpy(mu_main).to(dev), origin=torch.from_numpy(origin).to(dev),
                  inputs_in_original_order=True)
    rp.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rp.out).view(np.uint32), np.concatenate(want).view(np.uint32))
    with pytest.raises(B.DqError):                                                  # needs origin
        B.Replay(ctx, topo, B.DQ_DYNAMIQ, [to_dev(g, dev) for g in orig], J, counts, n_buckets=buckets,
                 inputs_in_original_order=True)


def test_pipelined_hops_on_a_gathered_local(dev):
    n, n_sg, first, block_sg = 4, [6, 9, 4, 3], 40, 5
    total = sum(n_sg)
    rng = np.random.default_rng(33)
    orig = [make_local(rng, (total + 3) * 256, "bf16") for _ in range(2)]
    idx = rng.permutation(total + 3)[:total].astype(np.int32)
    mu = (rng.standard_normal(total) * 2e-4).astype(np.float32)
    orc, ctx = O.Oracle(n, seed=15), B.Context(n, seed=15)
    gch = B.make_chunk(first, n_sg)
    blocks = block_chunks(n_sg, block_sg, first)
    msgs = [None] * len(blocks)
    for hop in range(2):
        g = orig[hop].reshape(-1, 256)[idx].reshape(-1)
        for i, (lo, hi, ch) in enumerate(blocks):
            x = np.ascontiguousarray(g[lo * 256:hi * 256])
            msgs[i] = orc.compress(ch, hop, x, mu[lo:hi]) if hop == 0 else orc.dar_hop(ch, hop, msgs[i], x, mu[lo:hi])
    want = np.concatenate([np.concatenate([m, np.zeros((-len(m)) % 256, np.uint8)]) for m in msgs])
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    wire = None
    for hop in range(2):
        wire = B.dq_dar_hop_pipelined(ctx, wire, to_dev(orig[hop], dev), gch, hop, block_sg, s1, s2,
                                      mu=torch.from_numpy(mu).to(dev), sg_index=torch.from_numpy(idx).to(dev))
        s1.synchronize()
    assert np.array_equal(host(wire), want)


@pytest.mark.parametrize("all_gather", [False, True])
def test_chain_replay_writes_the_restored_result(dev, all_gather):
    from oracle import pp_oracle as P
    n, n_sg = 5, [6, 9, 4, 3]
    total = sum(n_sg)
    rng = np.random.default_rng(55 + all_gather)
    sl = [make_local(rng, total * 256, "bf16") for _ in range(n)]
    mu = (rng.standard_normal(total) * 2e-4).astype(np.float32)
    mu[total - n_sg[3]:] = 0
    origin = rng.permutation(total).astype(np.int32)
    orc, ctx = O.Oracle(n, seed=8), B.Context(n, seed=8)
    och = O.make_chunk(9, n_sg)
    msg = orc.compress(och, 0, sl[0], mu)
    for i in range(1, n - 1):
        msg = orc.dar_hop(och, i, msg, sl[i], mu)
    res = orc.decompress(och, msg, sl[n - 1], mu)
    if all_gather:
        res = orc.decompress(och, orc.compress(och, n - 1, res))
    want = P.restore(res, np.argsort(origin).astype(np.uint32), mu, n)
    rc = B.Replay(ctx, B.DQ_CHAIN, B.DQ_DYNAMIQ, [to_dev(s, dev) for s in sl], total, [n_sg], first_sg=9,
                  all_gather=all_gather, mu=torch.from_numpy(mu).to(dev), origin=torch.from_numpy(origin).to(dev))
    rc.run()
    torch.cuda.synchronize()
    assert np.array_equal(host(rc.out).view(np.uint32), want.view(np.uint32))
    with pytest.raises(B.DqError):          # a chain's slices are chunks, not buckets: no gathered inputs
        B.Replay(ctx, B.DQ_CHAIN, B.DQ_DYNAMIQ, [to_dev(s, dev) for s in sl], total, [n_sg], first_sg=9,
                 origin=torch.from_numpy(origin).to(dev), inputs_in_original_order=True)


def test_replay_can_be_captured_in_a_graph(dev):
    """The replay only launches kernels (no allocation, no memset, no synchronisation), so a caller may
    capture it in a HIP graph; every replay of the graph, with eager work between, gives the eager bytes."""
    n, J = 8, 64
    counts = [[10, 30, 20, 4]]
    rng = np.random.default_rng(91)
    grads = [to_dev(make_local(rng, J * 256, "bf16"), dev) for _ in range(n)]
    mu = torch.from_numpy((rng.standard_normal(J) * 2e-4).astype(np.float32)).to(dev)
    origin = torch.from_numpy(rng.permutation(J).astype(np.int32)).to(dev)
    ctx = B.Context(n, seed=4)
    rp = B.Replay(ctx, B.DQ_BUTTERFLY, B.DQ_DYNAMIQ, grads, J, counts, all_gather=True, mu=mu, origin=origin,
                  inputs_in_original_order=True)
    rp.run()
    torch.cuda.synchronize()
    ref = rp.out.clone()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        rp.run()                                        # warm the capture stream
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        rp.run_steps(0, rp.n_steps)
    torch.cuda.synchronize()
    for i in range(4):
        rp.out.fill_(float(i))                          # eager work between the replays
        scratch_probe = (grads[i] * 2).sum()            # a library reduction too
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(rp.out, ref), f"graph replay {i}"
        assert torch.isfinite(scratch_probe)
