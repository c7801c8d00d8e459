"""The paper's large-scale simulation (Section 6.2) inside one GPU's HBM: a compressed all-reduce
over n simulated workers -- up to the paper's data-parallel dimension of 8,192 with 32,768
super-groups per worker, 137 GB of bf16 gradients resident at once -- on the synthetic workload
of its appendix, reporting the compression error (vNMSE) and the time of the hop replay.

    python -m paper_2602_08923_amd.large_scale --workers 1024 --sg 32768 --bits 8.5 --topology ring

Gradients are drawn twice from the same seeds (once for the statistics and the exact sum, once
to stay resident), so that only one copy per worker is ever held.  There is no reorder pass and no
restore pass: the replay's kernels gather super-groups from the original tensors and the last one
writes the original order."""
import argparse
import json
import math
import time

import torch

from . import allreduce as A
from . import binding as B
from . import prep, workloads


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workers", type=int, default=1024)
    ap.add_argument("--sg", type=int, default=32768, help="super-groups per worker (a multiple of --workers)")
    ap.add_argument("--bits", type=float, default=8.5)
    ap.add_argument("--topology", choices=["ring", "butterfly"], default="ring")
    ap.add_argument("--codec", choices=["dynamiq", "mxfp8"], default="dynamiq")
    ap.add_argument("--max-width", type=int, default=16, choices=[8, 16], help="W = {2,4,8} or {2,4,8,16} (the paper's setting here)")
    ap.add_argument("--g4", type=float, default=1.3, help="1 + 2 eps^2 of the 4-bit level set")
    ap.add_argument("--g8", type=float, default=1.02, help="1 + 2 eps^2 of the 8-bit level set")
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    n, J = args.workers, args.sg
    if J % n:
        raise SystemExit("--sg must be a multiple of --workers")
    dev = torch.device("cuda:0")
    topo = B.DQ_RING if args.topology == "ring" else B.DQ_BUTTERFLY
    M = workloads.mixture_magnitudes(J, seed=args.seed, device=dev)
    entries = J * 256
    t0 = time.perf_counter()
    truth = torch.zeros(entries, dtype=torch.float64, device=dev)
    dynamiq = args.codec == "dynamiq"
    if dynamiq:
        mu_all = torch.empty((n, J), dtype=torch.float32, device=dev)
        F_all = torch.empty((n, J), dtype=torch.float32, device=dev)
    for w in range(n):                                   # pass 1: statistics and the exact sum
        g = workloads.draw_mixture(M, w, seed=args.seed)
        truth += g.double()
        if dynamiq:
            B.dq_sg_stats(g, mu_all[w], F_all[w])
    by_width = None
    if dynamiq:
        mu, F = B.dq_stats_combine(mu_all, F_all)
        del mu_all, F_all
        budget = int(math.floor(prep.code_bits(args.bits) * J))
        widths, pos, counts = B.dq_allocate(F, J, budget, max_width=args.max_width)
        by_width = [[int(v) for v in counts.cpu().tolist()[0][:4]]]
        mu_main, origin = B.dq_reorder_mean(mu, pos, J, counts, with_origin=True)
    resident = []
    for w in range(n):                                   # pass 2: the resident gradients
        g = workloads.draw_mixture(M, w, seed=args.seed)
        resident.append(g)                               # original order: the kernels gather through `origin`
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ctx = B.Context(n, seed=1234 + args.seed, g4=args.g4, g8=args.g8)
    codec = B.DQ_DYNAMIQ if dynamiq else B.DQ_MXFP8_E4M3
    # the schedule's last launch writes the original order with the means added back (the restore, fused)
    rp = B.Replay(ctx, topo, codec, resident, J, by_width, all_gather=True, mu=mu_main if dynamiq else None,
                  origin=origin if dynamiq else None, inputs_in_original_order=dynamiq)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    rp.run()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    out = rp.out
    err = A.vnmse(out, truth)
    print(json.dumps({
        "workers": n, "super_groups_per_worker": J, "entries_per_worker": entries, "topology": args.topology,
        "codec": args.codec, "budget_bits": args.bits if dynamiq else 8.25, "g4": args.g4, "g8": args.g8, "sg_by_width_2_4_8_16": by_width[0] if by_width else None,
        "vNMSE": err, "gradient_GB_resident": round(n * entries * 2 / 1e9, 2),
        "scratch_GB": round(rp.scratch.numel() / 1e9, 2), "replay_steps": rp.n_steps,
        "seconds": {"generate_stats": round(t1 - t0, 2), "build_schedule": round(t2 - t1, 2),
                    "replay": round(t3 - t2, 4)},
        "entry_hops_per_second": round(n * entries / (t3 - t2) / 1e9, 2),
    }))


if __name__ == "__main__":
    main()
