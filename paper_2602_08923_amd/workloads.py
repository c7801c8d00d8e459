"""Seeded synthetic gradient generators and the five benchmark configurations.

This module holds no arithmetic of the codec: it only draws the inputs that both
the HIP path and the CPU oracle are run on (the same bits go to both), with the
shapes and value distributions of the workloads the paper trains on (dense
LLM fine-tuning gradients cut into 25 MB DDP buckets, Section 5 "Workloads"),
which are not available here.  Everything is a pure function of (config, worker,
bucket) through a seeded torch.Generator on the requested device; small cases
are drawn on the CPU and uploaded, large ones are drawn in HBM and the slices
the oracle checks are copied back.
"""
from dataclasses import dataclass, field

import numpy as np
import torch

S = 256  # super-group size (Section 5, "configuration")
BUCKET = 13_107_200  # entries in one 25 MB bf16 DDP bucket


@dataclass
class Workload:
    name: str
    topology: str            # "ring", "butterfly" or "chain" (one chunk's ring path)
    n_workers: int
    entries: int             # entries per worker per bucket (chain: entries of the one chunk)
    dtype: str               # "f32" or "bf16"
    budget_bits: float       # b-bar, overall bits per coordinate
    dist: str                # "normal", "outliers", "layers", "student_t"
    n_buckets: int = 1
    codec: str = "dynamiq"
    seed_base: int = 0
    extra: dict = field(default_factory=dict)


CONFIGS = {
    1: Workload("cfg1_ring4_f32_2p20", "ring", 4, 1 << 20, "f32", 5.0, "normal", seed_base=0),
    2: Workload("cfg2_ring8_bf16_25MB", "ring", 8, BUCKET, "bf16", 4.0, "outliers", seed_base=2000),
    3: Workload("cfg3_ring8_bf16_25MB_mx", "ring", 8, BUCKET, "bf16", 8.25, "outliers", codec="mx", seed_base=2000),
    4: Workload("cfg4_bfly16_bf16_1p3B", "butterfly", 16, BUCKET, "bf16", 3.0, "layers", n_buckets=100,
                seed_base=4000),
    5: Workload("cfg5_chain64_bf16_125M", "chain", 64, 125_000_192, "bf16", 5.0, "student_t", seed_base=5000),
}


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def layer_sigmas(n_entries_total, seed):
    """Per-tensor standard deviations for the 'layers' distribution: a generic
    GPT-style shape table (embedding 50304x2048, then 24 blocks of 2048x6144,
    2048x2048, 2048x8192, 8192x2048) flattened; each tensor draws one sigma
    log-uniformly from [1e-5, 1e-2].  Returns (boundaries, sigmas) as numpy arrays."""
    shapes = [50304 * 2048]
    for _ in range(24):
        shapes += [2048 * 6144, 2048 * 2048, 2048 * 8192, 8192 * 2048]
    bounds = np.minimum(np.cumsum(shapes), n_entries_total)
    rng = np.random.Generator(np.random.PCG64(seed))
    sig = 10.0 ** rng.uniform(-5.0, -2.0, size=len(shapes))
    if bounds[-1] < n_entries_total:  # whatever is left takes one more tensor
        bounds = np.append(bounds, n_entries_total)
        sig = np.append(sig, 10.0 ** rng.uniform(-5.0, -2.0))
    return bounds, sig


def draw(wl: Workload, worker: int, bucket: int = 0, device="cpu", entries=None):
    """Worker `worker`'s gradient for bucket `bucket`, as a torch tensor of wl.dtype
    on `device`.  `entries` overrides wl.entries (tests use shortened buckets)."""
    n = wl.entries if entries is None else entries
    seed = wl.seed_base + 1000 * bucket + worker if wl.seed_base else worker
    g = _gen(device, seed)
    if wl.dist == "normal":
        x = torch.randn(n, generator=g, device=device, dtype=torch.float32) * 1e-3
    elif wl.dist == "outliers":
        x = torch.randn(n, generator=g, device=device, dtype=torch.float32) * 1e-3
        k = max(1, n // 1000)  # 0.1 % of the entries, chosen uniformly, scaled x100
        idx = torch.randint(0, n, (k,), generator=g, device=device)
        x[idx] *= 100.0
    elif wl.dist == "layers":
        total = wl.entries * wl.n_buckets
        bounds, sig = layer_sigmas(total, wl.seed_base)
        lo = bucket * wl.entries
        pos = np.arange(lo, lo + n, S)  # sigma is constant within a super-group-aligned run
        sg_sigma = sig[np.searchsorted(bounds, pos, side="right").clip(max=len(sig) - 1)]
        scale = torch.from_numpy(sg_sigma.astype(np.float32)).to(device).repeat_interleave(S)[:n]
        x = torch.randn(n, generator=g, device=device, dtype=torch.float32) * scale
    elif wl.dist == "student_t":
        # Student-t with nu = 3: z / sqrt(chi2_3 / 3), chi2_3 as a sum of three squared normals
        z = torch.randn(n, generator=g, device=device, dtype=torch.float32)
        c = torch.zeros(n, device=device, dtype=torch.float32)
        for _ in range(3):
            c += torch.randn(n, generator=g, device=device, dtype=torch.float32) ** 2
        x = z / torch.sqrt(c / 3.0) * 1e-3
    else:
        raise ValueError(wl.dist)
    return x if wl.dtype == "f32" else x.to(torch.bfloat16)


# Section 6.2 / Appendix "Synthesizing data": the magnitude M of a super-group follows a mixture
# of two LogNormal laws fitted to measured per-super-group norms (weights, mu, sigma of ln M as
# printed with the paper's fit for K = 2); every coordinate of every worker is N(0, M^2 / 256).
MIXTURE = ((0.79, -3.99, 1.22), (0.21, -16.41, 4.63))


def mixture_magnitudes(n_sg, seed=0, device="cpu"):
    """One magnitude per super-group, shared by all workers (float32 tensor)."""
    g = _gen(device, 7_000_000 + seed)
    pick = torch.rand(n_sg, generator=g, device=device)
    z = torch.randn(n_sg, generator=g, device=device)
    first = pick < MIXTURE[0][0]
    mu = torch.where(first, torch.tensor(MIXTURE[0][1], device=device), torch.tensor(MIXTURE[1][1], device=device))
    sd = torch.where(first, torch.tensor(MIXTURE[0][2], device=device), torch.tensor(MIXTURE[1][2], device=device))
    return torch.exp(mu + sd * z).to(torch.float32)


def draw_mixture(magnitudes, worker, seed=0, dtype=torch.bfloat16, out=None):
    """Worker `worker`'s gradient for the given super-group magnitudes: i.i.d. N(0, M^2/256)
    inside each super-group, rounded to `dtype`.  `out` (same dtype) is filled in place if given."""
    device = magnitudes.device
    n_sg = magnitudes.numel()
    g = _gen(device, 7_100_000 + 100_000 * seed + worker)
    x = torch.randn(n_sg, S, generator=g, device=device, dtype=torch.float32)
    x *= (magnitudes / 16.0).unsqueeze(1)
    x = x.reshape(-1)
    if out is not None:
        out.copy_(x)
        return out
    return x.to(dtype)


def to_numpy(t: torch.Tensor):
    """Host copy as numpy: float32 stays float32, bfloat16 becomes its uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
