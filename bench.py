#!/usr/bin/env python3
"""Benchmark of the DynamiQ hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: the full
reduce-scatter hop replay of the chosen workload (compress, every DAR hop, the final
decompress-accumulate) for all simulated workers, inputs resident in HBM.  The default
workload is benchmark configuration 2: 8-worker ring over one 25 MB bf16 DDP bucket per
worker (13,107,200 entries, N(0,1e-3) with 0.1 % x100 outliers), DynamiQ at ~4 bits/entry.

Prints ONE JSON line.  `value` = gradient bytes processed per second over the whole replay
(entries handled by every hop x sizeof(gradient dtype) / time).  `roofline` prices the
dominant kernel (the DAR hop) by its algorithmic bytes per entry / its launch duration
measured with HIP events on the launch stream.  `cpu_baseline` times the CPU oracle on a
bounded sample of the same workload on one host core.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# HBM bytes per DAR launch from two `rocprofv3 --pmc` runs of this script (FETCH_SIZE, then
# WRITE_SIZE; KiB per dispatch), each scaled by what the same counter reads for a plain copy of
# 2^30 bytes on the same box: FETCH_SIZE counts half the bytes read (x2.0), WRITE_SIZE all of
# them (x1.0).  Key: (workload, codec).  The summary with the commands sits in profiles/.
MEASURED_TRAFFIC_BYTES = {
    (2, 0): int((16260.5 * 2.0 + 6238.4 * 1.0) * 1024),
}
# Vector-ALU wave instructions per DAR launch, from `rocprofv3 --pmc SQ_INSTS_VALU` on the same
# command (profiles/); one wave instruction is 64 lane operations.
MEASURED_VALU_WAVE_INSTR = {
    (2, 0): 5_818_511,
}
# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz: lane operations per second the vector ALUs can issue
VALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12
HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E published peak


def algorithmic_bytes_per_entry(codec, counts_total, n_sg_total, dtype_bytes, kind):
    """Bytes the method itself must move per entry for one launch kind.
    DynamiQ: codes (2/4/8 bits) + 16 u8 group scales + one bf16 SG scale per 256 entries;
    MX: 8/6/4-bit codes + one E8M0 byte per 32 entries."""
    if codec == 0:
        packed = (64 * counts_total[0] + 128 * counts_total[1] + 256 * counts_total[2] + 18 * n_sg_total) / (256.0 * n_sg_total)
        dtype_bytes = dtype_bytes + 4.0 / 256.0  # one fp32 mean per super-group read beside the local entries
    else:
        packed = {1: 8, 2: 6, 3: 4}[codec] / 8.0 + 1.0 / 32.0
    if kind == "compress":
        return dtype_bytes + packed
    if kind == "dar":
        return dtype_bytes + 2 * packed
    return packed + dtype_bytes + 4.0  # decompress-accumulate: packed + local in, fp32 out


def _cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=2, choices=[1, 2, 3, 5], help="benchmark configuration number")
    ap.add_argument("--mx-format", type=int, default=1, choices=[1, 2, 3], help="config 3 only: 1 FP8, 2 FP6, 3 FP4")
    ap.add_argument("--entries", type=int, default=None, help="override entries per worker (multiple of 256*workers)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle baseline (0 = skip)")
    ap.add_argument("--no-prepost", action="store_true",
                    help="skip the context timings of the steps before and after the main stage")
    ap.add_argument("--no-mean", action="store_true",
                    help="run the main stage without per-super-group means (the default subtracts them, Section 3.1)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy, as the known-size reference row for HBM counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (N simulated workers share its HBM); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_08923_amd import binding as B
    from paper_2602_08923_amd import prep, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    wl = workloads.CONFIGS[args.workload]
    n = wl.n_workers
    entries = args.entries or wl.entries
    codec = args.mx_format if wl.codec == "mx" else B.DQ_DYNAMIQ
    dtype_bytes = 4 if wl.dtype == "f32" else 2
    topo = {"ring": B.DQ_RING, "butterfly": B.DQ_BUTTERFLY, "chain": B.DQ_CHAIN}[wl.topology]

    # ---- inputs (untimed): draw in HBM, allocate widths from F_j, reorder by width
    grads = [workloads.draw(wl, w, 0, device=dev, entries=entries) for w in range(n)]
    if codec == B.DQ_DYNAMIQ:
        F = prep.squared_norms(grads)
        widths = prep.allocate(F, wl.budget_bits)
        perm, counts = prep.reorder_plan(widths, 1 if wl.topology == "chain" else n)
        grads = [prep.apply_reorder(g, perm) for g in grads]
        del F, widths
    else:
        counts = [entries // 256, 0, 0]
    n_sg = entries // 256
    ctx = B.Context(n, seed=20260208, round=0)
    # the per-super-group means the main stage subtracts (Section 3.1), from the library's own
    # statistics of the reordered gradients (untimed: the statistics exchange precedes the main stage)
    mu_main = None
    if codec == B.DQ_DYNAMIQ and not args.no_mean:
        mu_all = torch.empty((n, n_sg), dtype=torch.float32, device=dev)
        F_all = torch.empty((n, n_sg), dtype=torch.float32, device=dev)
        for w in range(n):
            B.dq_sg_stats(grads[w], mu_all[w], F_all[w])
        mu_main, _ = B.dq_stats_combine(mu_all, F_all)
        del mu_all, F_all
    rp = B.Replay(ctx, topo, codec, grads, n_sg, [counts], mu=mu_main)
    n_steps = rp.n_steps
    infos = [rp.step_info(i) for i in range(n_steps)]
    hop_entries = sum(a + b for _, a, b in infos)  # entries handled by all launches of one replay

    # ---- timed region: exactly K replays.  Each replay is enqueued as [compress][all DAR hop
    # steps][final decompress-accumulate]; HIP events on the launch stream bracket the run of
    # DAR launches, so the dominant kernel's duration comes from the same region as `value`.
    dar_steps = [i for i, (k, _, _) in enumerate(infos) if k == 1]
    first_dar = dar_steps[0] if dar_steps else n_steps
    n_dar = len(dar_steps)
    assert dar_steps == list(range(first_dar, first_dar + n_dar))

    def replay(ev=None):
        rp.run_steps(0, first_dar)
        if ev:
            ev[0].record()
        rp.run_steps(first_dar, n_dar)
        if ev:
            ev[1].record()
        rp.run_steps(first_dar + n_dar, n_steps - first_dar - n_dar)

    for _ in range(args.warmup):
        replay()
    # Every `every`-th replay of the timed region carries the event bracket (two event records and
    # two more calls into the library cost about 15 us of a 125 us replay); the others are one call.
    every = max(1, min(8, args.steps // 8))
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range((args.steps + every - 1) // every)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % every == 0:
            replay(events[i // every])
        else:
            rp.run_steps(0, n_steps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = hop_entries * dtype_bytes / (ms_per_step * 1e-3) / 1e9

    kind_names = {0: "compress", 1: "dar", 2: "decompress_accumulate", 3: "dar+decompress_accumulate"}
    if dar_steps:
        dar_ms = float(np.mean([a.elapsed_time(b) for a, b in events])) / n_dar
        dar_entries = infos[dar_steps[0]][1]
        bpe = algorithmic_bytes_per_entry(codec, counts, n_sg, dtype_bytes, "dar")
        achieved = bpe * dar_entries / (dar_ms * 1e-3) / 1e9
    else:
        dar_ms, dar_entries, bpe, achieved = float("nan"), 0, 0.0, 0.0

    # ---- context only (outside the timed region): every hop step timed on its own
    acc = np.zeros(n_steps)
    reps = max(1, min(args.steps, 20))
    for _ in range(reps):
        acc += np.array(rp.run(timed=True))
    step_ms = acc / reps
    per_kind = {}
    for i, (k, a, b) in enumerate(infos):
        per_kind.setdefault(kind_names[k], []).append(float(step_ms[i]))
    roofline = {
        "bound": "hbm", "kernel": "dq_dar_hop" if codec == 0 else "dq_mx_dar_hop",
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBPS, 4),
        "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, codec)),
        "algorithmic_bytes_per_entry": bpe, "entries_per_launch": dar_entries,
        "avg_launch_us": round(dar_ms * 1e3, 2),
        "gradient_GBps_per_dar_hop": round(dar_entries * dtype_bytes / (dar_ms * 1e-3) / 1e9, 1) if dar_steps else None,
        "launches_per_replay": n_dar,
        # the kernel is bound by vector-ALU issue, not by HBM: the same launch priced against the issue rate
        "alu_view": None if (args.workload, codec) not in MEASURED_VALU_WAVE_INSTR or not dar_steps else {
            "bound": "alu", "unit": "T lane-op/s", "peak": round(VALU_PEAK_TLANEOPS, 2),
            "achieved": round(MEASURED_VALU_WAVE_INSTR[(args.workload, codec)] * 64 / (dar_ms * 1e-3) / 1e12, 2),
            "frac": round(MEASURED_VALU_WAVE_INSTR[(args.workload, codec)] * 64 / (dar_ms * 1e-3) / 1e12 / VALU_PEAK_TLANEOPS, 4),
            "valu_wave_instructions_per_launch": MEASURED_VALU_WAVE_INSTR[(args.workload, codec)]},
        "timing": f"HIP events on the launch stream bracketing the consecutive DAR launches of every {every}-th replay inside the timed region ({len(events)} brackets)",
    }

    # ---- context only: the steps before and after the main stage on this workload's shape
    # (statistics of every worker, their combination, allocation, reorder of every worker,
    # restore of the result), each timed with events over `reps` runs
    prepost = None
    if codec == 0 and not args.no_prepost and wl.topology != "chain":
        import math
        raw = [workloads.draw(wl, w, 0, device=dev, entries=entries) for w in range(n)]
        mu_all = torch.empty((n, n_sg), dtype=torch.float32, device=dev)
        F_all = torch.empty((n, n_sg), dtype=torch.float32, device=dev)
        budget = int(math.floor(prep.code_bits(wl.budget_bits) * n_sg))
        re_out = torch.empty_like(raw[0])
        final = torch.empty(entries, dtype=torch.float32, device=dev)
        state = {}

        def f_stats():
            for w in range(n):
                B.dq_sg_stats(raw[w], mu_all[w], F_all[w])

        def f_combine():
            state["mu"], state["F"] = B.dq_stats_combine(mu_all, F_all)

        def f_alloc():
            state["w"], state["pos"], state["counts"] = B.dq_allocate(state["F"], n_sg, budget)

        def f_mean():
            state["mu_main"] = B.dq_reorder_mean(state["mu"], state["pos"], n_sg, state["counts"])

        def f_reorder():
            for w in range(n):
                B.dq_reorder(raw[w], state["pos"], n_sg, out=re_out)

        def f_restore():
            B.dq_restore(rp.out, state["pos"], n_sg, n, mu_main=state["mu_main"], out=final)

        def timed(fn):
            fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            b.synchronize()
            return a.elapsed_time(b) * 1e3 / reps

        t_stats, t_comb, t_alloc, t_mean = timed(f_stats), timed(f_combine), timed(f_alloc), timed(f_mean)
        t_reo, t_res = timed(f_reorder), timed(f_restore)
        c = state["counts"].cpu().numpy()[0]
        # the same reduce-scatter from the ORIGINAL tensors: reorder pass + replay + restore pass against
        # one replay whose kernels gather on the way in and scatter (with n * mu) on the way out
        mm, origin = B.dq_reorder_mean(state["mu"], state["pos"], n_sg, state["counts"], with_origin=True)
        gpu_counts = [[int(v) for v in c[:4]]]
        re_all = [B.dq_reorder(raw[w], state["pos"], n_sg) for w in range(n)]
        rp_sep = B.Replay(ctx, topo, codec, re_all, n_sg, gpu_counts, mu=mm)
        rp_fused = B.Replay(ctx, topo, codec, raw, n_sg, gpu_counts, mu=mm, origin=origin, inputs_in_original_order=True)

        def f_three_passes():
            for w in range(n):
                B.dq_reorder(raw[w], state["pos"], n_sg, out=re_all[w])
            rp_sep.run()
            B.dq_restore(rp_sep.out, state["pos"], n_sg, n, mu_main=mm, out=final)

        t_three, t_fused = timed(f_three_passes), timed(rp_fused.run)
        same = bool(torch.equal(final, rp_fused.out))
        del re_all, rp_sep, rp_fused
        prepost = {
            "stats_us": round(t_stats, 1), "stats_GBps": round(n * entries * dtype_bytes / t_stats / 1e3, 1),
            "combine_us": round(t_comb, 1), "allocate_us": round(t_alloc, 1), "reorder_mean_us": round(t_mean, 1),
            "reorder_us": round(t_reo, 1), "reorder_GBps": round(n * entries * 2 * dtype_bytes / t_reo / 1e3, 1),
            "restore_us": round(t_res, 1), "restore_GBps": round(entries * 8 / t_res / 1e3, 1),
            "sg_by_width_2_4_8_gpu_allocation": [int(c[0]), int(c[1]), int(c[2])],   # W = {2,4,8}: c[3] (16-bit) is 0
            "reorder_replay_restore_us": {"three_passes": round(t_three, 1), "fused_into_the_replay": round(t_fused, 1),
                                          "same_bits": same},
            "note": "all workers per figure (stats and reorder: one launch per worker); GB/s = bytes read + written",
        }
        del raw, re_out, final

    if args.calibrate_copy:  # 2^30 bytes read + 2^30 bytes written by one copy kernel
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- CPU oracle on a bounded sample of the same workload, one host core
    cpu = None
    if args.cpu_seconds > 0:
        from oracle import dq_oracle as O
        sample_sg = min(n_sg // (1 if wl.topology == "chain" else n), 2048)
        if codec == 0:
            # super-groups of each width in the proportion the whole bucket has them
            edges = np.cumsum([0] + counts)
            cw = [int(round(sample_sg * counts[w] / n_sg)) for w in range(3)]
            cw[1] += sample_sg - sum(cw)
            och = O.make_chunk(0, cw)
            orc = O.Oracle(n, seed=20260208, round=0)
            pick = torch.cat([torch.arange(int(edges[w]), int(edges[w]) + cw[w]) for w in range(3)]).to(dev)
            sl = [workloads.to_numpy(g.reshape(-1, 256)[pick].reshape(-1)) for g in grads[:3]]
            omu = None if mu_main is None else mu_main[pick].cpu().numpy()
        else:
            sl = [workloads.to_numpy(g[:sample_sg * 256]) for g in grads[:3]]
        if codec == 0:
            msg = orc.compress(och, 0, sl[0], omu)
        else:
            msg = O.mx_compress(codec, sl[0])
        hops, t_cpu = 0, 0.0
        c0 = time.perf_counter()
        while True:
            if codec == 0:
                msg = orc.dar_hop(och, 1 + (hops & 1), msg, sl[1 + (hops & 1)], omu)
            else:
                msg = O.mx_dar_hop(codec, msg, sl[1 + (hops & 1)])
            hops += 1
            t_cpu = time.perf_counter() - c0
            if t_cpu >= args.cpu_seconds or hops >= 10000:
                break
        cpu_entries = hops * sample_sg * 256
        cpu = {
            "value": round(cpu_entries * dtype_bytes / t_cpu / 1e9, 5), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{hops} DAR hops over {sample_sg} super-groups ({sample_sg * 256} entries) of worker slices 1-2, "
                      f"{t_cpu:.1f} s single-threaded C oracle",
            "ns_per_entry_hop": round(t_cpu / cpu_entries * 1e9, 2),
            "host_cpus_visible": os.cpu_count(), "host_cpu_model": _cpu_model(),
        }

    out = {
        "metric": "DAR-hop gradient GB/s", "value": round(value, 2), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "topology": wl.topology, "simulated_workers": n, "entries_per_worker": entries,
                   "grad_dtype": wl.dtype, "codec": "dynamiq" if codec == 0 else {1: "mxfp8_e4m3", 2: "mxfp6_e3m2", 3: "mxfp4_e2m1"}[codec],
                   "budget_bits": wl.budget_bits if codec == 0 else None, "sg_by_width_2_4_8": counts if codec == 0 else None,
                   "mean_subtraction": mu_main is not None,
                   "hop_steps_per_replay": n_steps, "entries_all_hops": hop_entries},
        "roofline": roofline,
        "prepost": prepost,
        "cpu_baseline": cpu,
        "step_ms_by_kind": {k: round(float(np.mean(v)), 5) for k, v in per_kind.items()},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
