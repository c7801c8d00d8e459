"""The whole simulated all-reduce of one bucket set on one GPU, as a sequence of boundary calls:
statistics -> their combination -> bit allocation -> [reorder ->] hop replay (reduce-scatter with
the means subtracted where the gradients enter, optionally the all-gather) [-> restore]
(Sections 3.1-3.4); by default the reorder and the restore happen inside the replay's kernels
(gathered loads, scattered stores).  Host glue only:
every step runs in the library's kernels.  Also the error measure the paper reports."""
import math

import torch

from . import binding as B
from . import prep


def vnmse(estimate, truth):
    """||estimate - truth||^2 / ||truth||^2 in float64 (the paper's vNMSE, Section 5)."""
    e = estimate.double() - truth.double()
    return float((e * e).sum() / (truth.double() ** 2).sum())


def true_sum(worker_grads):
    acc = torch.zeros(worker_grads[0].numel(), dtype=torch.float64, device=worker_grads[0].device)
    for g in worker_grads:
        acc += g.double()
    return acc


def simulated_allreduce(worker_grads, budget_bits, topology=B.DQ_RING, codec=B.DQ_DYNAMIQ, seed=0, round=0,
                        all_gather=True, subtract_mean=True, n_sg_bucket=None, g4=1.3, g8=1.02, max_width=8,
                        independent_rounding=False, uniform_width=None, fused_restore=True, fused_reorder=True):
    """Returns (sum estimate in the original order, float32; info dict).
    worker_grads: one tensor per simulated worker (same length, float32 or bfloat16, a whole
    number of buckets of n_sg_bucket super-groups; default: one bucket).  MX codecs skip the
    statistics, allocation and reorder (they have none) and ignore budget_bits.
    max_width: 8 for W = {2,4,8}, 16 for W = {2,4,8,16}.  uniform_width (2, 4 or 8): no allocation,
    every super-group at that width (the baseline the variable allocation is compared with).
    fused_restore: the replay's last launch writes the original order with the means added back
    (dq_replay_desc.origin); False: a separate dq_restore pass does.  fused_reorder (with
    fused_restore): the kernels gather the super-groups from the original tensors, there is no
    dq_reorder pass; False: every worker's tensor is reordered first.  Same bytes either way."""
    n = len(worker_grads)
    entries = worker_grads[0].numel()
    n_sg = entries // 256
    J = n_sg_bucket or n_sg
    if entries % 256 or n_sg % J or J % n:
        raise B.DqError("buckets must hold a multiple of n_workers super-groups of 256 entries")
    nb = n_sg // J
    ctx = B.Context(n, seed=seed, round=round, g4=g4, g8=g8, independent_rounding=independent_rounding)
    if codec != B.DQ_DYNAMIQ:
        rp = B.Replay(ctx, topology, codec, worker_grads, J, n_buckets=nb, all_gather=all_gather)
        rp.run()
        return rp.out, {"replay_steps": rp.n_steps}
    dev = worker_grads[0].device
    mu_all = torch.empty((n, n_sg), dtype=torch.float32, device=dev)
    F_all = torch.empty((n, n_sg), dtype=torch.float32, device=dev)
    for w, g in enumerate(worker_grads):
        B.dq_sg_stats(g, mu_all[w], F_all[w])
    mu, F = B.dq_stats_combine(mu_all, F_all)
    if not subtract_mean:
        mu = None
    counts = None
    if uniform_width is None:
        budget = int(math.floor(prep.code_bits(budget_bits) * J))
        widths, pos, counts = B.dq_allocate(F, J, budget, max_width=max_width)
        by_width = [[int(v) for v in row[:4]] for row in counts.cpu().tolist()]
    else:
        pos = torch.arange(J, dtype=torch.int32, device=dev).repeat(nb)
        row = [0, 0, 0, 0]
        row[{2: 0, 4: 1, 8: 2, 16: 3}[uniform_width]] = J
        by_width = [row] * nb
        if uniform_width == 16:
            mu = None                                    # uncompressed super-groups are not normalized
    mu_main, origin = B.dq_reorder_mean(mu, pos, J, counts, with_origin=True)
    gather = fused_reorder and fused_restore
    inputs = worker_grads if gather else [B.dq_reorder(g, pos, J) for g in worker_grads]
    rp = B.Replay(ctx, topology, B.DQ_DYNAMIQ, inputs, J, by_width, n_buckets=nb, all_gather=all_gather,
                  mu=mu_main, origin=origin if fused_restore else None, inputs_in_original_order=gather)
    rp.run()
    out = rp.out if fused_restore else B.dq_restore(rp.out, pos, J, n, mu_main=mu_main)
    return out, {"sg_by_width": by_width, "replay_steps": rp.n_steps}
