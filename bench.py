#!/usr/bin/env python3
"""Benchmark of the DynamiQ hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: the full
reduce-scatter hop replay of the chosen workload (compress, every DAR hop, every
decompress-accumulate) for all simulated workers, inputs resident in HBM.  The default
workload is benchmark configuration 2: 8-worker ring over one 25 MB bf16 DDP bucket per
worker (13,107,200 entries, N(0,1e-3) with 0.1 % x100 outliers), DynamiQ at ~4 bits/entry.

Prints ONE JSON line.  `value` = gradient bytes processed per second over the whole replay
(entries handled by every hop x sizeof(gradient dtype) / time).  `roofline` prices the
dominant kernel (the DAR hop) by its algorithmic bytes per entry / its launch duration
measured with HIP events on the launch stream inside the timed region, and carries
`copy_ceiling`: a streaming probe with the DAR hop's read : write ratio, run in the same
process.  `roofline_by_config` repeats the DAR measurement on the other configurations
(3: the three MX formats, 4: the 100-bucket butterfly, 5: the 64-worker chain), each set up
and torn down in turn.  `cpu_baseline` times the CPU oracle on a bounded sample of the
headline workload on one host core.
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Figures that only a profiler run can give, each from a summary under profiles/ made with this
# script (the summary names its command).  Key: (workload, codec).  Workloads without an entry
# print null: nothing is carried over from another configuration.
#   traffic: HBM bytes per DAR launch from two `rocprofv3 --pmc` runs (FETCH_SIZE, then WRITE_SIZE;
#            KiB per dispatch), each scaled by what the same counter reads for a plain copy of 2^30
#            bytes on the same box: FETCH_SIZE counts half the bytes read (x2.0), WRITE_SIZE all (x1.0).
#   valu:    vector-ALU wave instructions per DAR launch (SQ_INSTS_VALU); one is 64 lane operations.
MEASURED = {
    (2, 0): {"traffic": int((16261.1 * 2.0 + 6228.8 * 1.0) * 1024), "valu": 5_244_460, "profile": "profiles/dq_dar_hop_cfg2_pmc.txt"},
}
# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz: lane operations per second the vector ALUs can issue
VALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12
HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E published peak
KIND_NAMES = {0: "compress", 1: "dar", 2: "decompress_accumulate", 3: "dar+decompress_accumulate"}
CODEC_NAMES = {0: "dynamiq", 1: "mxfp8_e4m3", 2: "mxfp6_e3m2", 3: "mxfp4_e2m1"}


def packed_bytes_per_entry(codec, counts_total, n_sg_total):
    """DynamiQ: codes (2/4/8 bits) + 16 u8 group scales + one bf16 SG scale per 256 entries;
    MX: 8/6/4-bit codes + one E8M0 byte per 32 entries."""
    if codec == 0:
        return (64 * counts_total[0] + 128 * counts_total[1] + 256 * counts_total[2] + 18 * n_sg_total) / (256.0 * n_sg_total)
    return {1: 8, 2: 6, 3: 4}[codec] / 8.0 + 1.0 / 32.0


def algorithmic_bytes_per_entry(codec, counts_total, n_sg_total, local_bytes, kind, with_mean):
    """Bytes the method itself must move per entry for one launch kind (local_bytes: 2 for a bf16
    gradient, 4 for fp32 gradients or an fp32 keep-buffer)."""
    packed = packed_bytes_per_entry(codec, counts_total, n_sg_total)
    if codec == 0 and with_mean:
        local_bytes = local_bytes + 4.0 / 256.0  # one fp32 mean per super-group read beside the local entries
    if kind == "compress":
        return local_bytes + packed
    if kind == "dar":
        return local_bytes + 2 * packed
    return packed + local_bytes + 4.0  # decompress-accumulate: packed + local in, fp32 out


def _cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return None


class Workload:
    """One configuration set up in HBM (untimed): gradients drawn, widths allocated from F_j,
    super-groups reordered by width, per-super-group means from the library's own statistics
    kernels, the hop schedule prepared."""

    def __init__(self, number, mx_format, dev, entries=None, use_mean=True, seed=20260208):
        import torch
        from paper_2602_08923_amd import binding as B
        from paper_2602_08923_amd import prep, workloads
        self.number = number
        wl = self.wl = workloads.CONFIGS[number]
        n = self.n = wl.n_workers
        self.entries = entries or wl.entries
        self.codec = mx_format if wl.codec == "mx" else B.DQ_DYNAMIQ
        self.dtype_bytes = 4 if wl.dtype == "f32" else 2
        topo = {"ring": B.DQ_RING, "butterfly": B.DQ_BUTTERFLY, "chain": B.DQ_CHAIN}[wl.topology]
        nb = self.n_buckets = wl.n_buckets
        d = self.entries
        self.n_sg = d // 256
        self.ctx = B.Context(n, seed=seed, round=0)
        counts_all, mus = [], []
        if nb == 1:
            grads = [workloads.draw(wl, w, 0, device=dev, entries=d) for w in range(n)]
            if self.codec == B.DQ_DYNAMIQ:
                F = prep.squared_norms(grads)
                widths = prep.allocate(F, wl.budget_bits)
                perm, counts = prep.reorder_plan(widths, 1 if wl.topology == "chain" else n)
                grads = [prep.apply_reorder(g, perm) for g in grads]
                del F, widths, perm
            else:
                counts = [self.n_sg, 0, 0]
            counts_all.append(counts)
        else:  # many buckets per worker, each allocated and reordered on its own
            grads = [torch.empty(d * nb, dtype=torch.bfloat16 if wl.dtype == "bf16" else torch.float32, device=dev)
                     for _ in range(n)]
            for b in range(nb):
                g = [workloads.draw(wl, w, b, device=dev, entries=d) for w in range(n)]
                re, counts, _ = prep.prepare_bucket(g, wl.budget_bits, n)
                counts_all.append(counts)
                for w in range(n):
                    grads[w][b * d:(b + 1) * d] = re[w]
                del g, re
        self.grads = grads
        self.counts_all = counts_all
        self.counts_total = [sum(c[k] for c in counts_all) for k in range(3)]
        self.mu = None
        if self.codec == B.DQ_DYNAMIQ and use_mean:
            J = self.n_sg * nb
            mu_all = torch.empty((n, J), dtype=torch.float32, device=dev)
            F_all = torch.empty((n, J), dtype=torch.float32, device=dev)
            for w in range(n):
                B.dq_sg_stats(grads[w], mu_all[w], F_all[w])
            self.mu, _ = B.dq_stats_combine(mu_all, F_all)
            del mu_all, F_all
        self.rp = B.Replay(self.ctx, topo, self.codec, grads, self.n_sg, counts_all, n_buckets=nb, mu=self.mu)
        self.infos = [self.rp.step_info(i) for i in range(self.rp.n_steps)]
        self.hop_entries = sum(a + b for _, a, b in self.infos)  # entries handled by all launches of one replay
        # the schedule as a list of calls; a DAR launch is a step of kind 1 or launch 0 of a step of kind 3
        self.calls = []
        for i, (k, a, b) in enumerate(self.infos):
            if k == 3:
                self.calls += [("launch", i, 0, True, a), ("launch", i, 1, False, b)]
            else:
                self.calls.append(("step", i, 0, k == 1, a if k == 1 else b))
        # butterfly steps after the second one read fp32 keep-buffers instead of the gradient
        self.dar_local_bytes = [self.dtype_bytes if (wl.topology != "butterfly" or i <= 1) else 4
                                for (_, i, _, is_dar, _) in self.calls if is_dar]
        self.dar_with_mean = [self.mu is not None and (wl.topology != "butterfly" or i <= 1)
                              for (_, i, _, is_dar, _) in self.calls if is_dar]

    def replay(self, events=None):
        """Enqueue one whole replay.  events: a list that receives (start, end) event pairs, one per
        maximal run of consecutive DAR launches."""
        import torch
        rp = self.rp
        if events is None:
            rp.run_steps(0, rp.n_steps)
            return
        in_run = False
        for what, step, launch, is_dar, _ in self.calls:
            if is_dar and not in_run:
                a = torch.cuda.Event(enable_timing=True)
                a.record()
                in_run = True
            if not is_dar and in_run:
                b = torch.cuda.Event(enable_timing=True)
                b.record()
                events.append((a, b))
                in_run = False
            if what == "step":
                rp.run_steps(step, 1)
            else:
                rp.run_launch(step, launch)
        if in_run:
            b = torch.cuda.Event(enable_timing=True)
            b.record()
            events.append((a, b))

    def measure(self, steps, warmup):
        """Time exactly `steps` replays; every `every`-th carries the event brackets of its DAR launches."""
        import numpy as np
        import torch
        for _ in range(warmup):
            self.replay()
        # two event records and extra calls into the library cost a few us per bracket: most replays run plain
        every = max(1, min(8, steps // 8))
        brackets = []
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.replay(brackets if i % every == 0 else None)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / steps
        value = self.hop_entries * self.dtype_bytes / (ms_per_step * 1e-3) / 1e9
        dar = [(e, lb, wm) for (_, _, _, is_dar, e), lb, wm in
               zip([c for c in self.calls if c[3]], self.dar_local_bytes, self.dar_with_mean)]
        n_dar = len(dar)
        res = {"ms_per_step": ms_per_step, "value": value, "n_dar": n_dar, "bracketed_replays": (steps + every - 1) // every,
               "every": every}
        if n_dar:
            total_ms = float(sum(a.elapsed_time(b) for a, b in brackets)) / res["bracketed_replays"]  # per replay
            total_bytes = sum(e * algorithmic_bytes_per_entry(self.codec, self.counts_total, self.n_sg * self.n_buckets, lb, "dar", wm)
                              for e, lb, wm in dar)
            res.update({
                "dar_us": total_ms * 1e3 / n_dar,
                "dar_entries": sum(e for e, _, _ in dar) / n_dar,
                "dar_bytes_per_entry": total_bytes / sum(e for e, _, _ in dar),
                "dar_achieved_GBps": total_bytes / (total_ms * 1e-3) / 1e9,
                "dar_gradient_GBps": sum(e * lb for e, lb, _ in dar) / (total_ms * 1e-3) / 1e9,
            })
        return res

    def step_times(self, reps):
        import numpy as np
        acc = np.zeros(self.rp.n_steps)
        for _ in range(reps):
            acc += np.array(self.rp.run(timed=True))
        per_kind = {}
        for i, (k, _, _) in enumerate(self.infos):
            per_kind.setdefault(KIND_NAMES[k], []).append(float(acc[i] / reps))
        return {k: round(float(np.mean(v)), 5) for k, v in per_kind.items()}

    def close(self):
        import torch
        self.rp.close()
        self.rp = None
        self.grads = None
        self.mu = None
        gc.collect()
        torch.cuda.empty_cache()


def copy_ceiling(ctx, read_bytes, write_bytes, dev, reps=40):
    """The streaming probe at the DAR launch's read and write sizes: once cycling through as many
    distinct input regions as the replay's DAR launches read between two visits of the same data
    (same footprint, so the 256 MB Infinity Cache helps or not as it does for the replay), once over
    inputs of 4 GB (HBM only)."""
    import torch
    from paper_2602_08923_amd import binding as B
    if read_bytes > (1 << 30):  # a probe launch of 1 GiB is in the streaming regime already: keep the ratio, cap the size
        write_bytes = int(write_bytes * float(1 << 30) / read_bytes)
        read_bytes = 1 << 30
    rb, wb = (read_bytes // 16) * 16, max(16, (write_bytes // 16) * 16)
    out = {"read_bytes": rb, "write_bytes": wb, "read_write_ratio": round(rb / wb, 2)}
    for name, regions in (("same_footprint_GBps", 8), ("hbm_only_GBps", max(8, min(256, (4 << 30) // rb)))):
        src = torch.empty(regions * rb, dtype=torch.uint8, device=dev)
        src.view(torch.int32).random_(0, 1 << 30)
        dst = torch.empty(2 * wb, dtype=torch.uint8, device=dev)
        def launches(count):
            for i in range(count):
                B.dq_stream_probe(ctx, src[(i % regions) * rb:(i % regions + 1) * rb], dst[(i & 1) * wb:((i & 1) + 1) * wb])

        launches(regions)  # warm-up: one pass over everything
        torch.cuda.synchronize()
        n = max(reps, regions)
        best = float("inf")
        for _ in range(5):  # the ceiling is the best of five batches (the first ones still see clocks ramping)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            launches(n)
            b.record()
            b.synchronize()
            best = min(best, a.elapsed_time(b) * 1e3 / n)
        us = best
        out[name] = round((rb + wb) / us / 1e3, 1)
        out[name.replace("_GBps", "_launch_us")] = round(us, 2)
        del src, dst
    out["frac_of_peak"] = round(out["same_footprint_GBps"] / HBM_PEAK_GBPS, 4)
    return out


def prepost_context(W, reps):
    """Context only: the steps before and after the main stage on this workload's shape (statistics of
    every worker, their combination, allocation, reorder of every worker, restore of the result), each
    timed with events over `reps` runs; whether the allocation of the next bucket hides beside the
    replay of this one (two default-priority streams); reorder + replay + restore as three passes
    against one replay that gathers on the way in and scatters on the way out."""
    import math
    import torch
    from paper_2602_08923_amd import binding as B
    from paper_2602_08923_amd import prep, workloads
    wl, n, n_sg, entries, dev = W.wl, W.n, W.n_sg, W.entries, W.grads[0].device
    dtype_bytes = W.dtype_bytes
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
        B.dq_restore(W.rp.out, state["pos"], n_sg, n, mu_main=state["mu_main"], out=final)

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

    # does the allocation of bucket k+1 hide beside the replay of bucket k?  `reps` replays on the current
    # stream and `reps` allocations on a second stream of the same (default) priority, forked and joined
    # ONCE (a cross-stream dependency costs tens of microseconds: per round it would swamp the answer)
    side = torch.cuda.Stream()
    t_replay = timed(W.rp.run)

    def both_total():
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(reps):
                f_alloc()
        for _ in range(reps):
            W.rp.run()
        torch.cuda.current_stream().wait_stream(side)
        b.record()
        b.synchronize()
        return a.elapsed_time(b) * 1e3 / reps

    both_total()
    t_both = both_total()

    def hidden(t_a, t_b):
        return round(max(0.0, min(1.0, (t_replay + t_a - t_b) / min(t_a, t_replay))), 3)

    # the same reduce-scatter from the ORIGINAL tensors: reorder pass + replay + restore pass against
    # one replay whose kernels gather on the way in and scatter (with n * mu) on the way out
    mm, origin = B.dq_reorder_mean(state["mu"], state["pos"], n_sg, state["counts"], with_origin=True)
    gpu_counts = [[int(v) for v in c[:4]]]
    re_all = [B.dq_reorder(raw[w], state["pos"], n_sg) for w in range(n)]
    topo = {"ring": B.DQ_RING, "butterfly": B.DQ_BUTTERFLY, "chain": B.DQ_CHAIN}[wl.topology]
    rp_sep = B.Replay(W.ctx, topo, W.codec, re_all, n_sg, gpu_counts, mu=mm)
    rp_fused = B.Replay(W.ctx, topo, W.codec, raw, n_sg, gpu_counts, mu=mm, origin=origin, inputs_in_original_order=True)

    def f_three_passes():
        for w in range(n):
            B.dq_reorder(raw[w], state["pos"], n_sg, out=re_all[w])
        rp_sep.run()
        B.dq_restore(rp_sep.out, state["pos"], n_sg, n, mu_main=mm, out=final)

    t_three, t_fused = timed(f_three_passes), timed(rp_fused.run)
    same = bool(torch.equal(final, rp_fused.out))
    rp_sep.close()
    rp_fused.close()
    return {
        "stats_us": round(t_stats, 1), "stats_GBps": round(n * entries * dtype_bytes / t_stats / 1e3, 1),
        "combine_us": round(t_comb, 1), "allocate_us": round(t_alloc, 1), "reorder_mean_us": round(t_mean, 1),
        "reorder_us": round(t_reo, 1), "reorder_GBps": round(n * entries * 2 * dtype_bytes / t_reo / 1e3, 1),
        "restore_us": round(t_res, 1), "restore_GBps": round(entries * 8 / t_res / 1e3, 1),
        "sg_by_width_2_4_8_gpu_allocation": [int(c[0]), int(c[1]), int(c[2])],   # W = {2,4,8}: c[3] (16-bit) is 0
        "allocate_beside_replay_us": {"replay_alone": round(t_replay, 1), "allocate_alone": round(t_alloc, 1),
                                      "both_on_two_streams": round(t_both, 1),
                                      "allocation_hidden_frac": hidden(t_alloc, t_both),
                                      "note": "per repetition, from one fork and one join around 20 repetitions on each stream"},
        "reorder_replay_restore_us": {"three_passes": round(t_three, 1), "fused_into_the_replay": round(t_fused, 1),
                                      "same_bits": same},
        "note": "all workers per figure (stats and reorder: one launch per worker); GB/s = bytes read + written",
    }


def cpu_oracle_baseline(W, seconds):
    """The CPU oracle's DAR hop, single-threaded, on a bounded sample of the headline workload."""
    import numpy as np
    import torch
    from oracle import dq_oracle as O
    from paper_2602_08923_amd import workloads
    n, n_sg, counts, codec, grads = W.n, W.n_sg, W.counts_all[0], W.codec, W.grads
    dev = grads[0].device
    sample_sg = min(n_sg // (1 if W.wl.topology == "chain" else n), 2048)
    if codec == 0:
        # super-groups of each width in the proportion the whole bucket has them
        edges = np.cumsum([0] + counts)
        cw = [int(round(sample_sg * counts[w] / n_sg)) for w in range(3)]
        cw[1] += sample_sg - sum(cw)
        och = O.make_chunk(0, cw)
        orc = O.Oracle(n, seed=20260208, round=0)
        pick = torch.cat([torch.arange(int(edges[w]), int(edges[w]) + cw[w]) for w in range(3)]).to(dev)
        sl = [workloads.to_numpy(g.reshape(-1, 256)[pick].reshape(-1)) for g in grads[:3]]
        omu = None if W.mu is None else W.mu[pick].cpu().numpy()
        msg = orc.compress(och, 0, sl[0], omu)
    else:
        sl = [workloads.to_numpy(g[:sample_sg * 256]) for g in grads[:3]]
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
        if t_cpu >= seconds or hops >= 10000:
            break
    cpu_entries = hops * sample_sg * 256
    return {
        "value": round(cpu_entries * W.dtype_bytes / t_cpu / 1e9, 5), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"{hops} DAR hops over {sample_sg} super-groups ({sample_sg * 256} entries) of worker slices 1-2, "
                  f"{t_cpu:.1f} s single-threaded C oracle",
        "ns_per_entry_hop": round(t_cpu / cpu_entries * 1e9, 2),
        "host_cpus_visible": os.cpu_count(), "host_cpu_model": _cpu_model(),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=2, choices=[1, 2, 3, 4, 5], help="benchmark configuration number")
    ap.add_argument("--mx-format", type=int, default=1, choices=[1, 2, 3], help="config 3 only: 1 FP8, 2 FP6, 3 FP4")
    ap.add_argument("--entries", type=int, default=None, help="override entries per worker (multiple of 256*workers)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle baseline (0 = skip)")
    ap.add_argument("--no-prepost", action="store_true",
                    help="skip the context timings of the steps before and after the main stage")
    ap.add_argument("--no-by-config", action="store_true",
                    help="skip the DAR measurements on the other configurations (roofline_by_config)")
    ap.add_argument("--no-copy-ceiling", action="store_true", help="skip the streaming probe")
    ap.add_argument("--no-mean", action="store_true",
                    help="run the main stage without per-super-group means (the default subtracts them, Section 3.1)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy, as the known-size reference row for HBM counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (N simulated workers share its HBM); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")

    # ---- the headline workload: untimed set-up, then the timed region of exactly K replays
    W = Workload(args.workload, args.mx_format, dev, entries=args.entries, use_mean=not args.no_mean)
    m = W.measure(args.steps, args.warmup)
    codec = W.codec
    reps = max(1, min(args.steps, 20))
    step_ms_by_kind = W.step_times(reps)
    known = MEASURED.get((args.workload, codec), {}) if args.entries is None and not args.no_mean else {}
    roofline = {
        "bound": "hbm", "kernel": "dq_dar_hop" if codec == 0 else "dq_mx_dar_hop",
        "achieved": round(m.get("dar_achieved_GBps", 0.0), 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(m.get("dar_achieved_GBps", 0.0) / HBM_PEAK_GBPS, 4),
        "traffic": known.get("traffic"),
        "algorithmic_bytes_per_entry": m.get("dar_bytes_per_entry"), "entries_per_launch": m.get("dar_entries"),
        "avg_launch_us": round(m.get("dar_us", float("nan")), 2),
        "gradient_GBps_per_dar_hop": round(m.get("dar_gradient_GBps", 0.0), 1),
        "launches_per_replay": m["n_dar"],
        # the kernel is bound by vector-ALU issue, not by HBM: the same launch priced against the issue rate
        "alu_view": None if not known.get("valu") or not m["n_dar"] else {
            "bound": "alu", "unit": "T lane-op/s", "peak": round(VALU_PEAK_TLANEOPS, 2),
            "achieved": round(known["valu"] * 64 / (m["dar_us"] * 1e-6) / 1e12, 2),
            "frac": round(known["valu"] * 64 / (m["dar_us"] * 1e-6) / 1e12 / VALU_PEAK_TLANEOPS, 4),
            "valu_wave_instructions_per_launch": known["valu"]},
        "counters_from": known.get("profile") if known.get("traffic") or known.get("valu") else None,
        "timing": f"HIP events on the launch stream bracketing every run of consecutive DAR launches of every "
                  f"{m['every']}-th replay inside the timed region ({m['bracketed_replays']} replays bracketed)",
    }
    if not args.no_copy_ceiling and m["n_dar"]:
        read_b = m["dar_entries"] * (m["dar_bytes_per_entry"] - packed_bytes_per_entry(codec, W.counts_total, W.n_sg * W.n_buckets))
        write_b = m["dar_entries"] * packed_bytes_per_entry(codec, W.counts_total, W.n_sg * W.n_buckets)
        roofline["copy_ceiling"] = copy_ceiling(W.ctx, int(read_b), int(write_b), dev)
        roofline["frac_of_copy_ceiling"] = round(m["dar_achieved_GBps"] / roofline["copy_ceiling"]["same_footprint_GBps"], 4)

    prepost = None
    if codec == 0 and not args.no_prepost and W.wl.topology != "chain" and W.n_buckets == 1:
        prepost = prepost_context(W, reps)

    if args.calibrate_copy:  # 2^30 bytes read + 2^30 bytes written by one copy kernel
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cpu = cpu_oracle_baseline(W, args.cpu_seconds) if args.cpu_seconds > 0 else None

    config = {"workload": W.wl.name, "topology": W.wl.topology, "simulated_workers": W.n, "entries_per_worker": W.entries,
              "buckets_per_worker": W.n_buckets, "grad_dtype": W.wl.dtype, "codec": CODEC_NAMES[codec],
              "budget_bits": W.wl.budget_bits if codec == 0 else None,
              "sg_by_width_2_4_8": W.counts_total if codec == 0 else None,
              "mean_subtraction": W.mu is not None,
              "hop_steps_per_replay": W.rp.n_steps, "entries_all_hops": W.hop_entries}
    W.close()
    del W

    # ---- the DAR hop on the other configurations, one after the other in this process
    by_config = None
    if not args.no_by_config:
        by_config = {}
        plan = [(3, 1, 20, 3), (3, 2, 20, 3), (3, 3, 20, 3), (4, 1, 3, 1), (5, 1, 5, 1), (2, 1, 30, 5)]
        for number, fmt, k, w in plan:
            if number == args.workload and (number != 3 or fmt == args.mx_format):
                continue
            try:
                X = Workload(number, fmt, dev)
                r = X.measure(k, w)
                name = X.wl.name + ("" if X.wl.codec != "mx" else "_" + CODEC_NAMES[X.codec])
                by_config[name] = {
                    "codec": CODEC_NAMES[X.codec], "dar_frac_of_hbm_peak": round(r["dar_achieved_GBps"] / HBM_PEAK_GBPS, 4),
                    "dar_achieved_GBps": round(r["dar_achieved_GBps"], 1), "avg_launch_us": round(r["dar_us"], 2),
                    "entries_per_launch": r["dar_entries"], "algorithmic_bytes_per_entry": round(r["dar_bytes_per_entry"], 6),
                    "launches_per_replay": r["n_dar"], "value_GBps": round(r["value"], 2), "ms_per_step": round(r["ms_per_step"], 4),
                    "steps": k, "warmup": w}
                if r["n_dar"]:
                    pk = packed_bytes_per_entry(X.codec, X.counts_total, X.n_sg * X.n_buckets)
                    cc = copy_ceiling(X.ctx, int(r["dar_entries"] * (r["dar_bytes_per_entry"] - pk)), int(r["dar_entries"] * pk), dev, reps=20)
                    by_config[name]["copy_ceiling_GBps"] = cc["same_footprint_GBps"]
                    by_config[name]["dar_frac_of_copy_ceiling"] = round(r["dar_achieved_GBps"] / cc["same_footprint_GBps"], 4)
                X.close()
                del X
            except Exception as e:  # a configuration that does not fit beside what else runs on the box: say so
                by_config[f"config_{number}_{CODEC_NAMES.get(fmt if number == 3 else 0)}"] = {"error": repr(e)[:200]}
                gc.collect()
                torch.cuda.empty_cache()

    out = {
        "metric": "DAR-hop gradient GB/s", "value": round(m["value"], 2), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(m["ms_per_step"], 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": config,
        "roofline": roofline,
        "roofline_by_config": by_config,
        "prepost": prepost,
        "cpu_baseline": cpu,
        "step_ms_by_kind": step_ms_by_kind,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
