#!/usr/bin/env python3
"""Benchmark of the shard hot path on one MI355X.

One "step" is one pass over every leg of the hot path at full workload size (see
tofu_workloads.py): two shard GEMMs, two shard convolutions, one shard weight gradient, the
halo region fetch and the two 8-way partition-n-reduce sums.  All inputs are resident in HBM
before the timed region; every leg is one call through the C ABI on torch's current stream.

Prints ONE JSON line.  `value` is the algorithmic FLOP of the contraction legs divided by the
wall time of the whole step (fetch and reduce legs included).  `legs` gives every leg's own
TFLOP/s or GB/s and roofline fraction from HIP events recorded between the legs; `roofline`
repeats the figures of the leg whose single kernel has the longest average duration.
"""
import argparse
import json
import os
import sys
import time

PEAK = {"mfma": (157.3, "TFLOP/s"), "hbm": (8000.0, "GB/s")}   # MI355X: fp32 matrix peak, HBM3E peak
ROOT = os.path.dirname(os.path.abspath(__file__))
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "all_legs_hbm_traffic.txt")


def read_traffic():
    """HBM-side bytes per launch of every leg, from the committed summary of the two hardware-counter
    runs (profiles/all_legs_hbm_traffic.txt): its `traffic_kib` lines give, per leg, the FETCH_SIZE and
    WRITE_SIZE KiB per dispatch summed over the leg's kernels and the factors that make each counter
    match that run's calibration copy.  -> {leg: bytes}; a leg without a line has no figure (None)."""
    out = {}
    try:
        for line in open(TRAFFIC_FILE):
            if not line.startswith("traffic_kib "):
                continue
            kv = dict(item.split("=", 1) for item in line.split()[1:])
            out[kv["leg"]] = round(1024.0 * (float(kv["fetch"]) * float(kv["fetch_scale"]) + float(kv["write"]) * float(kv["write_scale"])))
    except OSError:
        pass
    return out


LEG_KERNELS = {"conv_cout": "conv2d_kernel<64,256,4,1,4,8,balanced,3,3> + conv2d_segment_sum_kernel",
               "conv_cout_h": "conv2d_kernel<64,256,4,1,4,8,balanced,3,3> + conv2d_segment_sum_kernel",
               "wgrad_batch": "wgrad_kernel<128,32,fast,balanced,14,1,4> + wgrad_segment_sum_kernel",
               "gemm_ksplit": "matmul_kernel<KG=2,TA=false,TB=false,GUARDED=false>", "gemm_nsplit": "matmul_kernel<KG=2,TA=false,TB=false,GUARDED=false> + slice_sum_kernel"}
EXTRA_NOTES = {"conv_cout_h_fused": "replaces fetch_halo + conv_cout_h; reads the halo row out of the neighbour's whole 7-row block (no copy of it exists)",
               "gemm_ksplit_accumulate": "gemm_ksplit adding into a resident [128,32768] buffer (reduction fused into the epilogue)",
               "conv1d_cout": "the paper's conv1d (Fig. 1): 2048 channels, window 3, 512 outputs per row, batch 64, C_out/8 shard; filters [ci][co][dx] re-ordered inside the call",
               "wgrad_batch_accumulate": "wgrad_batch adding into a resident dW (reduction fused into the segment sum)",
               "lstm_cell_nsplit": "element-wise LSTM cell update on the N-split worker's 128 x 1024 hidden units (3.7 MB: launch-bound)",
               "dgrad_cout": "backward of conv_cout: partial dx[128,2560,14,14] from the C_out/8 blocks of dy and the filters (filter reversal included)",
               "gemm_dx_nsplit": "backward of gemm_nsplit: partial dX = dY_s . W_s^T (128x16384x4096), W_s read transposed in place",
               "gemm_dw_nsplit": "backward of gemm_nsplit: dW_s = X^T . dY_s (16384x4096x128), X read transposed in place"}
METRIC = "shard GEMM/conv TFLOP/s (% fp32 MFMA peak); partition-n-reduce GB/s (% HBM)"


def cpu_baseline(legs):
    """Time the fp64 oracle (OpenMP over outputs, all host cores) on a bounded part of every leg's output
    and extrapolate linearly to the leg's whole output box -> (aggregate object, {leg: per-leg entry})."""
    import numpy as np
    import oracle
    import tofu_synth as synth
    from oracle import regions as R
    oracle.build(force=False)
    flop, secs, parts, per_leg = 0.0, 0.0, [], {}

    def note(leg, t, n, total, what):
        per_leg[leg.name] = {"oracle_s": round(t * total / n, 3), "sample_s": round(t, 3), "sample": f"{n} of {total} {what}"}
        parts.append(f"{leg.name}: {n} {what}")

    for leg in legs:
        h = leg.host
        if h.get("kind") == "matmul":
            box = h["box"]
            n = 3 << 16 if "b_col0" in h else 3 << 18
            shape = [b[1] - b[0] for b in box]
            pts = synth.coords(900, 1, n, shape)
            k0, k1 = h["krange"]
            t = time.perf_counter()
            if "b_col0" in h:      # B is the worker's column block: local columns
                oracle.matmul_pts(h["A"], h["B"], pts, krange=(k0, k1))
            else:                  # B is the worker's row block: local rows, A columns shifted
                oracle.matmul_pts(np.ascontiguousarray(h["A"][:, k0:k1]), h["B"], pts)
            t = time.perf_counter() - t
            flop += 2.0 * n * (k1 - k0)
            note(leg, t, n, int(np.prod(shape)), "outputs")
        elif h.get("kind") == "conv2d":
            n = 3 << 17 if leg.name == "conv_cout" else 3 << 16
            shape = [b[1] - b[0] for b in h["box"]]
            lo = np.array([b[0] for b in h["box"]], dtype=np.int64)
            lo[1] = 0                                  # the worker's own filters: local output channels
            pts = synth.coords(900, 2, n, shape) + lo
            t = time.perf_counter()
            oracle.conv2d_pts(h["x"], h["w"], pts, stride=1, pad=1)
            t = time.perf_counter() - t
            flop += leg.work * n / float(np.prod(shape))
            note(leg, t, n, int(np.prod(shape)), "outputs")
        elif h.get("kind") == "wgrad":
            n = 3 << 16
            c = h["x"].shape[1]
            pts = synth.coords(900, 3, n, (c, c, 3, 3))
            t = time.perf_counter()
            oracle.wgrad_pts(h["x"], h["dy"], 3, 3, pts, stride=1, pad=1)
            t = time.perf_counter() - t
            flop += leg.work * n / float(c * c * 9)
            note(leg, t, n, c * c * 9, "outputs")
        elif h.get("kind") == "reduce" and "remote" in h:
            own = h["own"].cpu().numpy()
            order = h["remote"][:h["own_index"]] + [own] + h["remote"][h["own_index"]:]
            t = time.perf_counter()
            oracle.reduce(order)
            t = time.perf_counter() - t
            note(leg, t, own.size, own.size, "elements (the whole reduction)")
        elif h.get("kind") == "fetch" and h.get("x") is not None:
            x, box = h["x"], h["box"]
            h_cut = box[2][1] - 1                      # own rows [0, h_cut), the neighbour's block starts there
            own_box = [box[0], box[1], (0, h_cut), box[3]]
            nb_box = [box[0], box[1], (h_cut, x.shape[2]), box[3]]
            srcs = [(np.ascontiguousarray(x[:, :, :h_cut]), own_box), (np.ascontiguousarray(x[:, :, h_cut:]), nb_box)]
            t = time.perf_counter()
            R.fetch(box, srcs)
            t = time.perf_counter() - t
            n = int(np.prod([b[1] - b[0] for b in box]))
            note(leg, t, n, n, "elements (the whole region)")
        secs += per_leg.get(leg.name, {}).get("sample_s", 0.0)
    mfma_s = sum(per_leg[l.name]["sample_s"] for l in legs if l.bound == "mfma" and l.name in per_leg)
    agg = {"value": flop / mfma_s * 1e-12 if mfma_s > 0 else None, "unit": "TFLOP/s", "cores": oracle.threads(), "kind": "oracle",
           "cpu": cpu_model(), "seconds": round(secs, 3),
           "sample": "value = FLOP of the contraction samples / their seconds; seeded output coordinates, every term of each sum; "
                     "the streaming legs whole: " + "; ".join(parts)}
    return agg, per_leg


def attainable(torch, tofu, dev):
    """The probes of include/tofu_probe.h: what a register-only MFMA loop and plain streams reach on this
    GPU.  Every stream figure is cold: the launches rotate over buffer sets that together exceed the 256 MB
    last-level cache, and the time is that of `reps` launches back to back divided by `reps`."""
    sink = torch.zeros(64, dtype=torch.float32, device=dev)
    wgs, iters = 2048, 4096

    def timed(fns, reps):
        for f in fns:
            f()
        ms = []
        for _ in range(5):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for r in range(reps):
                fns[r % len(fns)]()
            b.record()
            b.synchronize()
            ms.append(a.elapsed_time(b) / reps)
        return sorted(ms)[2]
    out = {}
    t_mfma = timed([lambda: tofu.probe_mfma(sink, iters, wgs)], 1)
    out["mfma_loop_tflops"] = round(wgs * 4 * iters * 8 * 4096 / t_mfma * 1e-9, 1)
    big = [torch.empty(1 << 28, dtype=torch.float32, device=dev) for _ in range(3)]     # 1 GiB each
    gb = lambda nbytes, ms: round(nbytes / ms * 1e-6, 1)
    out["copy_1gib_gbs"] = gb(2 * big[0].numel() * 4, timed([lambda: tofu.probe_copy(big[1], big[0])], 2))
    out["copy_nontemporal_1gib_gbs"] = gb(2 * big[0].numel() * 4, timed([lambda: tofu.probe_stream(big[1], [big[0]])], 2))
    out["read_only_1gib_gbs"] = gb(big[0].numel() * 4, timed([lambda: tofu.probe_read(big[0], sink), lambda: tofu.probe_read(big[1], sink)], 4))
    del big
    # the streaming legs' own sizes and read:write mixes
    n_gate, n_dw, n_fetch = 128 * 32768, 1280 * 1280 * 9, 128 * 2560 * 8 * 14
    sets = [[torch.empty(n_dw, dtype=torch.float32, device=dev) for _ in range(9)] for _ in range(4)]
    mk = lambda n: [(lambda st: (lambda: tofu.probe_stream(st[8][:n], [t[:n] for t in st[:8]])))(st) for st in sets]
    out["stream_8to1_151mb_gbs"] = gb(9 * 4 * n_gate, timed(mk(n_gate), 16))
    out["stream_8to1_531mb_gbs"] = gb(9 * 4 * n_dw, timed(mk(n_dw), 8))
    del sets
    cp = [[torch.empty(n_fetch, dtype=torch.float32, device=dev) for _ in range(2)] for _ in range(3)]
    out["copy_nontemporal_294mb_gbs"] = gb(2 * 4 * n_fetch, timed([(lambda st: (lambda: tofu.probe_stream(st[1], [st[0]])))(st) for st in cp], 12))
    out["read_only_147mb_gbs"] = gb(4 * n_fetch, timed([(lambda st: (lambda: tofu.probe_read(st[0], sink)))(st) for st in cp] +
                                                       [(lambda st: (lambda: tofu.probe_read(st[1], sink)))(st) for st in cp], 12))
    return out


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--legs", type=str, default="", help="comma-separated subset of legs (default: all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also capture one step into a HIP graph and report its replay time (launch gaps removed)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch one plain elementwise copy of 256 MiB before the timed steps, so that a "
                         "hardware-counter run holds a kernel of known traffic to scale its counters by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs one worker's shard on ONE GPU; --gpus > 1 is not supported "
              "(other workers' partials and halo blocks are generated into the same GPU's HBM).", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1807_08887_amd as tofu
    import tofu_workloads
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback.", file=sys.stderr)
        sys.exit(2)
    tofu.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    peaks = attainable(torch, tofu, dev)
    torch.cuda.empty_cache()
    which = [s for s in args.legs.split(",") if s] or None
    names = which if which else list(tofu_workloads.STEP_LEGS) + list(tofu_workloads.EXTRA_LEGS)
    built = tofu_workloads.build(dev, names, keep_host=not args.no_cpu_baseline, cold_copies=True)
    legs = [l for l in built if l.name not in tofu_workloads.EXTRA_LEGS or which]
    extra_legs = [l for l in built if l not in legs]
    torch.cuda.synchronize()

    def step(events=None):
        for i, leg in enumerate(legs):
            if events is not None:
                events[i].record()
            leg.run()
        if events is not None:
            events[len(legs)].record()

    if args.calibration_copy:      # reads 2^26 floats, writes 2^26 floats (torch's vectorised elementwise kernel)
        cal_src = torch.empty(1 << 26, dtype=torch.float32, device=dev)    # contents do not matter
        cal_dst = torch.empty_like(cal_src)
        torch.mul(cal_src, 1.0, out=cal_dst)
        torch.cuda.synchronize()
        del cal_src, cal_dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # ---- the timed region: exactly `steps` steps, nothing but the legs' launches on the stream
    t0 = time.perf_counter()
    for s in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    # ---- the same steps again with a HIP event between the legs: the per-leg split (an event costs the
    # stream about 2.5 us, which these per-leg times therefore include and ms_per_step does not)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(legs) + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(ev[s])
    torch.cuda.synchronize()
    ms_per_step_events = (time.perf_counter() - t0) * 1e3 / args.steps

    traffic_of = read_traffic()
    per_step = [[ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(args.steps)] for i in range(len(legs))]
    leg_ms = [sum(t) / len(t) for t in per_step]
    leg_out = []
    for leg, ms, samples in zip(legs, leg_ms, per_step):
        peak, unit = PEAK[leg.bound]
        scale = 1e-9 if leg.bound == "mfma" else 1e-6           # FLOP/ms -> TFLOP/s, B/ms -> GB/s
        achieved = leg.work / ms * scale
        # ms = mean over the timed steps with events; median and min over the same launches.
        # Inside a step every leg finds its operands evicted by the other legs (a step moves about 3 GB): cache-cold.
        entry = {"leg": leg.name, "bound": leg.bound, "ms": round(ms, 4), "median_ms": round(sorted(samples)[len(samples) // 2], 4),
                 "min_ms": round(min(samples), 4), "achieved": round(achieved, 2), "unit": unit, "frac": round(achieved / peak, 4),
                 "traffic": traffic_of.get(leg.name)}
        if leg.conventional_flop:
            entry["conventional_tflops"] = round(leg.conventional_flop / ms * 1e-9, 2)
        leg_out.append(entry)
    # The streaming legs without the event: `reps` launches back to back on rotating copies of the operands
    # (cold, as in the step), time / reps = kernel + the gap to the next launch.  This is what the leg adds
    # to an uninstrumented step, so `achieved` / `frac` of these legs are taken from it; the event-bracketed
    # figures stay beside them as in_step_*.
    for leg, entry in zip(legs, leg_out):
        if leg.bound != "hbm" or not leg.cold:
            continue
        reps = 4 * len(leg.cold)
        for f in leg.cold:
            f()
        ms = []
        for _ in range(7):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for r in range(reps):
                leg.cold[r % len(leg.cold)]()
            b.record()
            b.synchronize()
            ms.append(a.elapsed_time(b) / reps)
        ms.sort()
        # the cache-warm figure beside it: the same launches on ONE operand set (what fits stays in the 256 MB last-level cache)
        warm = []
        for _ in range(5):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for r in range(reps):
                leg.cold[0]()
            b.record()
            b.synchronize()
            warm.append(a.elapsed_time(b) / reps)
        warm.sort()
        entry["cache_warm_ms"] = round(warm[2], 4)
        peak, unit = PEAK[leg.bound]
        entry.update({"in_step_ms": entry["ms"], "in_step_achieved": entry["achieved"], "in_step_frac": entry["frac"],
                      "ms": round(ms[3], 4), "min_ms": round(ms[0], 4), "median_ms": round(ms[3], 4),
                      "achieved": round(leg.work / ms[3] * 1e-6, 2), "frac": round(leg.work / ms[3] * 1e-6 / peak, 4),
                      "timing": f"{reps} launches back to back over {len(leg.cold)} rotating operand sets (cold), time / {reps}, median of 7 such runs; in_step_* = one launch between two HIP events inside the step; cache_warm_ms = the same on one operand set"})
    flop = sum(l.work for l in legs if l.bound == "mfma")
    # the roofline object repeats the contraction leg that takes longest (its fix-up kernel included)
    dom = max([e for e in leg_out if e["bound"] == "mfma"] or leg_out, key=lambda e: e["ms"])
    out = {
        "metric": METRIC, "value": round(flop / (ms_per_step * 1e-3) * 1e-12, 3), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "one step = every leg of the shard path at full size: " + ", ".join(l.name for l in legs),
                   "shapes": "LSTM gate GEMM 128x32768x16384 (8-way N and K shards); 3x3 conv 2560ch 14x14 batch 128 "
                             "(C_out/8 and C_out/8 x H/2 shards, halo fetch); 3x3 wgrad 1280ch 28x28 (batch/8 shard); 8-way reduces"},
        "roofline": {"kernel": dom["leg"] + ": " + LEG_KERNELS.get(dom["leg"], ""), "bound": dom["bound"], "achieved": dom["achieved"], "peak": PEAK[dom["bound"]][0],
                     "unit": dom["unit"], "frac": dom["frac"], "traffic": dom["traffic"]},
        "ms_per_step_with_leg_events": round(ms_per_step_events, 4),
        "attainable": peaks,
        "legs": leg_out,
    }
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        out["graph_replay_ms_per_step"] = round((time.perf_counter() - t0) * 1e3 / args.steps, 4)
    if extra_legs:
        # outside the step: the fused-fetch convolution and the backward GEMMs, timed right after
        # the steps (warm clocks)
        extras = []
        for leg in extra_legs:
            for _ in range(3):
                leg.run()
            e = [torch.cuda.Event(enable_timing=True) for _ in range(11)]
            for i in range(10):
                e[i].record()
                leg.run()
            e[10].record()
            torch.cuda.synchronize()
            ms = sorted(e[i].elapsed_time(e[i + 1]) for i in range(10))[5]
            peak, unit = PEAK[leg.bound]
            rate = leg.work / ms * (1e-9 if leg.bound == "mfma" else 1e-6)
            extras.append({"leg": leg.name, "bound": leg.bound, "ms": round(ms, 4), "achieved": round(rate, 2),
                           "unit": unit, "frac": round(rate / peak, 4),
                           "note": EXTRA_NOTES.get(leg.name, "") + "; median of 10 launches back to back"})
        out["extras"] = extras
    if not args.no_cpu_baseline:
        out["cpu_baseline"], per_leg = cpu_baseline(legs)
        for entry in leg_out:
            if entry["leg"] in per_leg:      # oracle seconds for the leg's whole output (sample, linearly extrapolated) beside the GPU time
                entry.update(per_leg[entry["leg"]])
                entry["oracle_over_gpu"] = round(per_leg[entry["leg"]]["oracle_s"] * 1e3 / entry["ms"], 1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
