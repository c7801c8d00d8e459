"""The paper's parametric study (Section 6.3: uniform levels -> non-uniform levels -> variable
bitwidth allocation -> correlated rounding) on synthetic gradients, as the error (vNMSE) of the whole
simulated all-reduce at the same communication budget.  Hierarchical scales cannot be switched
off in this library, so that row of the paper's table has no counterpart here.

    python -m paper_2602_08923_amd.ablation --workers 8 --sg 8192

With --scalability: the error against the worker count (Section 6.1: ring all-reduce, n = 2 .. 64),
DynamiQ at 5 bits beside the three MX formats, on the same synthetic workload.
"""
import argparse
import json

import torch

from . import allreduce as A
from . import binding as B
from . import workloads


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workers", type=int, default=8)
    ap.add_argument("--sg", type=int, default=8192)
    ap.add_argument("--topology", choices=["ring", "butterfly"], default="ring")
    ap.add_argument("--scalability", action="store_true", help="error against the worker count instead")
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    n, J = args.workers, args.sg
    topo = B.DQ_RING if args.topology == "ring" else B.DQ_BUTTERFLY
    if args.scalability:
        return scalability(J, topo, args.topology, dev)
    # every super-group at 4 bits costs 4 + 0.5 + 1/16 + 1/8 = 4.6875 bits per coordinate: the budget of all rows
    bits = 4.6875
    out = {}
    for name, grads in (
        ("lognormal-mixture magnitudes, Gaussian entries",
         [workloads.draw_mixture(workloads.mixture_magnitudes(J, seed=2, device=dev), w, seed=2) for w in range(n)]),
        ("lognormal-mixture magnitudes, 0.1 % of the entries x100",
         [_with_outliers(workloads.draw_mixture(workloads.mixture_magnitudes(J, seed=2, device=dev), w, seed=2), w) for w in range(n)]),
    ):
        truth = A.true_sum(grads)
        rows = {}
        kw = dict(topology=topo, seed=5)
        rows["uniform levels, 4 bits everywhere, independent rounding"] = A.vnmse(
            A.simulated_allreduce(grads, bits, uniform_width=4, g4=1.0001, g8=1.006, independent_rounding=True, **kw)[0], truth)
        rows["+ non-uniform levels"] = A.vnmse(
            A.simulated_allreduce(grads, bits, uniform_width=4, independent_rounding=True, **kw)[0], truth)
        rows["+ variable bitwidth allocation"] = A.vnmse(
            A.simulated_allreduce(grads, bits, independent_rounding=True, **kw)[0], truth)
        rows["+ correlated rounding"] = A.vnmse(A.simulated_allreduce(grads, bits, **kw)[0], truth)
        out[name] = rows
    print(json.dumps({"workers": n, "super_groups": J, "topology": args.topology, "budget_bits": bits, "vNMSE": out}, indent=1))


def scalability(J, topo, topo_name, dev):
    M = workloads.mixture_magnitudes(J, seed=2, device=dev)
    table = {}
    for n in (2, 4, 8, 16, 32, 64):
        grads = [workloads.draw_mixture(M, w, seed=2) for w in range(n)]
        truth = A.true_sum(grads)
        row = {"dynamiq_5_bits": A.vnmse(A.simulated_allreduce(grads, 5.0, topology=topo, seed=5)[0], truth)}
        for name, codec in (("mxfp8", B.DQ_MXFP8_E4M3), ("mxfp6", B.DQ_MXFP6_E3M2), ("mxfp4", B.DQ_MXFP4_E2M1)):
            row[name] = A.vnmse(A.simulated_allreduce(grads, 0.0, topology=topo, codec=codec)[0], truth)
        table[n] = row
    print(json.dumps({"super_groups": J, "topology": topo_name, "vNMSE_by_workers": table}, indent=1))


def _with_outliers(g, w):
    gen = torch.Generator(device=g.device)
    gen.manual_seed(9_000 + w)
    idx = torch.randint(0, g.numel(), (max(1, g.numel() // 1000),), generator=gen, device=g.device)
    g = g.clone()
    g[idx] *= 100.0
    return g


if __name__ == "__main__":
    main()
