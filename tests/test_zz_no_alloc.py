"""dq_dar_hop_pipelined_static -- the pipelined hop on the library's static staging array, for
callers that cannot allocate -- against dq_dar_hop_pipelined with a caller-owned stage: same wire
bytes, on two calls in a row (the second smaller, so it meets what the first left in the shared
array), and a clear refusal beyond the array's size.  Runs last: a failure here must not hide
the parity tests."""
import numpy as np
import pytest
import torch

from paper_2602_08923_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


def bf16_local(rng, n, dev):
    x = (rng.standard_normal(n) * np.repeat(10.0 ** rng.uniform(-4, -1, n // 16), 16)).astype(np.float32)
    return torch.from_numpy(x).to(dev).to(torch.bfloat16)


def hops(ctx, gch, block_sg, xs, mu, dev, static):
    """compress by worker 0, then DAR by workers 1 and 2, block-wise; returns the wire after each hop."""
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    wire, out = None, []
    for hop, x in enumerate(xs):
        if static:
            nxt = torch.zeros(B.dq_pipelined_wire_bytes(gch, block_sg), dtype=torch.uint8, device=dev)
            torch.cuda.synchronize()
            wire = B.dq_dar_hop_pipelined_static(ctx, wire, x, gch, hop, block_sg, s1, s2, nxt, mu=mu)
        else:
            torch.cuda.synchronize()
            wire = B.dq_dar_hop_pipelined(ctx, wire, x, gch, hop, block_sg, s1, s2, mu=mu)
        s1.synchronize()
        out.append(wire.cpu().numpy().copy())
    return out


def test_static_stage_matches_caller_stage_twice_in_a_row(dev):
    n = 8
    ctx = B.Context(n, seed=21, round=1)
    rng = np.random.default_rng(3)
    # first call: 4 widths, 11 blocks with a ragged last one; second call: fewer, smaller blocks
    for n_sg, block_sg, first in (([300, 411, 200, 90], 96, 5000), ([17, 30, 9, 3], 7, 2 ** 33 + 1)):
        total = sum(n_sg)
        gch = B.make_chunk(first, n_sg)
        assert B.dq_pipelined_stage_bytes(gch, block_sg) <= B.DQ_STATIC_STAGE_BYTES
        xs = [bf16_local(rng, total * 256, dev) for _ in range(3)]
        mu = torch.from_numpy((rng.standard_normal(total) * 1e-4).astype(np.float32)).to(dev)
        want = hops(ctx, gch, block_sg, xs, mu, dev, static=False)
        got = hops(ctx, gch, block_sg, xs, mu, dev, static=True)
        for hop, (g, w) in enumerate(zip(got, want)):
            assert np.array_equal(g, w), f"hop {hop} of the {total}-super-group chunk differs"
        assert want[0].any() and not np.array_equal(want[1], want[2])


def test_static_stage_rejects_blocks_beyond_its_size(dev):
    ctx = B.Context(4, seed=1)
    n_sg = [0, 0, 0, 20000]                                  # raw bf16: 512 B per super-group
    gch = B.make_chunk(0, n_sg)
    block_sg = 10000                                         # two blocks of 5 MB: beyond the 8 MiB array
    assert B.dq_pipelined_stage_bytes(gch, block_sg) > B.DQ_STATIC_STAGE_BYTES
    x = torch.zeros(sum(n_sg) * 256, dtype=torch.bfloat16, device=dev)
    wire = torch.zeros(B.dq_pipelined_wire_bytes(gch, block_sg), dtype=torch.uint8, device=dev)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    with pytest.raises(B.DqError, match="static scratch holds"):
        B.dq_dar_hop_pipelined_static(ctx, None, x, gch, 0, block_sg, s1, s2, wire)
    torch.cuda.synchronize()
    assert not wire.any()                                    # nothing was enqueued
    # the same chunk in blocks that fit goes through
    B.dq_dar_hop_pipelined_static(ctx, None, x, gch, 0, 4000, s1, s2,
                                  torch.zeros(B.dq_pipelined_wire_bytes(gch, 4000), dtype=torch.uint8, device=dev))
    s1.synchronize()
