"""Untimed set-up on either side of the hot path: bit allocation and reordering.

The hot path takes as inputs (a) how many super-groups use 2, 4 and 8 bits and
(b) every worker's bucket with its super-groups permuted so that equal widths are
contiguous, narrowest first (Section 3.5: "monotonically increasing bitwidth
order").  This module produces both from raw gradients, following Section 3.1
(F_j, the summed squared norms) and Appendix A (the three-width allocation rule
with one free offset u found by bisection).  It is float64 host/torch code used
by tests and the benchmark to prepare inputs for BOTH the HIP path and the CPU
oracle; it is not part of either.
"""
import math

import numpy as np
import torch

S = 256
GROUPS_PER_SG = 16
# Appendix A: z_j = K * log2(F_j) + u with K = 4 / log2(512/17); the thresholds
# T_{2,4} and T_{4,8} = (512/17) T_{2,4} (Section 3.2) sit at z = 4 and z = 8.
K_ALLOC = 4.0 / math.log2(512.0 / 17.0)


def code_bits(budget_bits):
    """Bits per coordinate left for the quantized representations: the budget minus
    the statistics all-reduce (32/S), the u8 group scales (8/16) and the bf16
    super-group scale (16/S)  (Section 3.5, "Communication overhead")."""
    return budget_bits - 32.0 / S - 8.0 / 16.0 - 16.0 / S


def squared_norms(worker_grads):
    """F_j = sum_i sum_{x in X_ij} x^2 in float64 (Section 3.1)."""
    F = None
    for g in worker_grads:
        f = g.to(torch.float64).reshape(-1, S).pow(2).sum(dim=1)
        F = f if F is None else F + f
    return F


def mean_per_super_group(worker_grads):
    """mu_j = (1/n) sum_i mean(X_ij) in float64, returned as float32 (Section 3.1): the means that
    tests and the benchmark hand to both the library and the oracle as an input."""
    acc = None
    for g in worker_grads:
        m = g.to(torch.float64).reshape(-1, 256).mean(dim=1)
        acc = m if acc is None else acc + m
    return (acc / len(worker_grads)).to(torch.float32)


def widths_for_offset(F, u):
    """q_j in {2,4,8}: 2 if z_j < 4, 4 if 4 <= z_j < 8, 8 if z_j >= 8 (Appendix A)."""
    z = K_ALLOC * torch.log2(F) + u  # F = 0 gives -inf, i.e. 2 bits
    q = torch.full_like(z, 2.0)
    q[z >= 4.0] = 4.0
    q[z >= 8.0] = 8.0
    return q


def allocate(F, budget_bits, iters=40):
    """Largest offset u (by bisection) whose allocation meets S*sum q_j <= d*code_bits.
    Returns an int64 tensor of widths per super-group."""
    target = code_bits(budget_bits) * F.numel()
    if target < 2.0 * F.numel():
        raise ValueError("budget leaves fewer than 2 code bits per coordinate")
    finite = F[F > 0]
    if finite.numel() == 0:
        return torch.full(F.shape, 2, dtype=torch.int64, device=F.device)
    lz = K_ALLOC * torch.log2(finite)
    lo = 4.0 - float(lz.max()) - 1.0   # everything at 2 bits
    hi = 8.0 - float(lz.min()) + 1.0   # everything at 8 bits
    if float(widths_for_offset(F, hi).sum()) <= target:
        return widths_for_offset(F, hi).to(torch.int64)
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        if float(widths_for_offset(F, mid).sum()) <= target:
            lo = mid
        else:
            hi = mid
    return widths_for_offset(F, lo).to(torch.int64)


def reorder_plan(widths, n_workers):
    """Stable permutation putting 2-bit super-groups first, then 4-bit, then 8-bit.
    Returns (perm, counts): reordered[j] = original[perm[j]], counts = [n2, n4, n8].
    The bucket must hold a multiple of n_workers super-groups (pad with zero
    super-groups beforehand)."""
    if widths.numel() % n_workers:
        raise ValueError("pad the bucket to a multiple of the worker count first")
    perm = torch.argsort(widths, stable=True)
    counts = [int((widths == b).sum()) for b in (2, 4, 8)]
    return perm, counts


def apply_reorder(grad, perm):
    return grad.reshape(-1, S)[perm].reshape(-1).contiguous()


def undo_reorder(reordered, perm):
    out = torch.empty_like(reordered).reshape(-1, S)
    out[perm] = reordered.reshape(-1, S)
    return out.reshape(-1)


def prepare_bucket(worker_grads, budget_bits, n_workers):
    """Allocation + reorder for one bucket.  Returns (reordered grads, counts, perm)."""
    F = squared_norms(worker_grads)
    widths = allocate(F, budget_bits)
    perm, counts = reorder_plan(widths, n_workers)
    return [apply_reorder(g, perm) for g in worker_grads], counts, perm


def chunk_counts(counts, n_chunks):
    """Width counts of each of n_chunks equal-length chunks of a reordered bucket."""
    total = sum(counts)
    m = total // n_chunks
    edges = [0, counts[0], counts[0] + counts[1], total]
    return [[max(0, min((i + 1) * m, edges[w + 1]) - max(i * m, edges[w])) for w in range(3)]
            for i in range(n_chunks)]
