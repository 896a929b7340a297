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
# HBM-side KiB per launch of every contraction leg (all kernels of the leg), from the two
# hardware-counter runs summarised in profiles/all_legs_hbm_traffic.txt: (FETCH_SIZE, WRITE_SIZE)
# per dispatch, each scaled by the factor that makes the same counter match the 256 MiB
# calibration copy of that run (2.0 for reads, 1.0 for writes).
TRAFFIC_KIB = {"conv_cout": (533973.0 + 32054.9, 64000.0 + 35703.7),        # conv2d_kernel + conv2d_segment_sum_kernel
               "conv_cout_h": (792886.0 + 24247.0, 48384.0 + 19040.2),
               "wgrad_batch": (1088130.0 + 63398.1, 126720.0 + 57727.8),    # wgrad_kernel + wgrad_segment_sum_kernel
               "gemm_ksplit": (149581.0, 16384.0),
               "gemm_nsplit": (149581.0 + 8211.0, 16384.0 + 2048.0)}        # matmul_kernel + slice_sum_kernel
TRAFFIC_SCALE = (2.0, 1.0)
LEG_KERNELS = {"conv_cout": "conv2d_kernel<64,256,4,1,4,8,balanced,3,3> + conv2d_segment_sum_kernel",
               "conv_cout_h": "conv2d_kernel<64,256,4,1,4,8,balanced,3,3> + conv2d_segment_sum_kernel",
               "wgrad_batch": "wgrad_kernel<128,32,fast,balanced,14,1,4> + wgrad_segment_sum_kernel",
               "gemm_ksplit": "matmul_kernel<128,64,32,2,2>", "gemm_nsplit": "matmul_kernel<128,64,32,2,2> + slice_sum_kernel"}
EXTRA_NOTES = {"conv_cout_h_fused": "replaces fetch_halo + conv_cout_h",
               "gemm_ksplit_accumulate": "gemm_ksplit adding into a resident [128,32768] buffer (reduction fused into the epilogue)",
               "conv1d_cout": "the paper's conv1d (Fig. 1): 2048 channels, window 3, 512 outputs per row, batch 64, C_out/8 shard; filters [ci][co][dx] re-ordered inside the call",
               "wgrad_batch_accumulate": "wgrad_batch adding into a resident dW (reduction fused into the segment sum)",
               "lstm_cell_nsplit": "element-wise LSTM cell update on the N-split worker's 128 x 1024 hidden units (3.7 MB: launch-bound)",
               "dgrad_cout": "backward of conv_cout: partial dx[128,2560,14,14] from the C_out/8 blocks of dy and the filters (filter reversal included)",
               "gemm_dx_nsplit": "backward of gemm_nsplit: partial dX = dY_s . W_s^T (128x16384x4096), W_s read transposed in place",
               "gemm_dw_nsplit": "backward of gemm_nsplit: dW_s = X^T . dY_s (16384x4096x128), X read transposed in place"}
METRIC = "shard GEMM/conv TFLOP/s (% fp32 MFMA peak); partition-n-reduce GB/s (% HBM)"


def cpu_baseline(legs):
    """Time the fp64 oracle on a bounded sample of the contraction legs' outputs (host cores)."""
    import numpy as np
    import oracle
    import tofu_synth as synth
    oracle.build(force=False)
    flop, secs, parts = 0.0, 0.0, []
    for leg in legs:
        h = leg.host
        if leg.bound != "mfma" or "kind" not in h:
            continue
        if h["kind"] == "matmul":
            box = h["box"]
            n = 3 << 17 if "b_col0" in h else 3 << 19
            pts = synth.coords(900, 1, n, [b[1] - b[0] for b in box])
            k0, k1 = h["krange"]
            t = time.perf_counter()
            if "b_col0" in h:      # B is the worker's column block: local columns
                oracle.matmul_pts(h["A"], h["B"], pts, krange=(k0, k1))
            else:                  # B is the worker's row block: local rows, A columns shifted
                oracle.matmul_pts(np.ascontiguousarray(h["A"][:, k0:k1]), h["B"], pts)
            secs += time.perf_counter() - t
            flop += 2.0 * n * (k1 - k0)
            parts.append(f"{leg.name}: {n} outputs")
        elif h["kind"] == "conv2d" and leg.name == "conv_cout":
            n = 3 << 18
            shape = [b[1] - b[0] for b in h["box"]]
            pts = synth.coords(900, 2, n, shape)
            t = time.perf_counter()
            oracle.conv2d_pts(h["x"], h["w"], pts, stride=1, pad=1)
            secs += time.perf_counter() - t
            flop += leg.work * n / float(np.prod(shape))
            parts.append(f"{leg.name}: {n} outputs")
        elif h["kind"] == "wgrad":
            n = 3 << 17
            c = h["x"].shape[1]
            pts = synth.coords(900, 3, n, (c, c, 3, 3))
            t = time.perf_counter()
            oracle.wgrad_pts(h["x"], h["dy"], 3, 3, pts, stride=1, pad=1)
            secs += time.perf_counter() - t
            flop += leg.work * n / float(c * c * 9)
            parts.append(f"{leg.name}: {n} outputs")
    return {"value": flop / secs * 1e-12 if secs > 0 else None, "unit": "TFLOP/s", "cores": oracle.threads(), "kind": "oracle",
            "cpu": cpu_model(),
            "seconds": round(secs, 3), "sample": "seeded output coordinates, every term of each sum: " + "; ".join(parts)}


def attainable(torch, tofu, dev):
    """The two probes of include/tofu_probe.h: what a register-only MFMA loop and a plain copy
    larger than the last-level cache reach on this GPU (median of 5 launches each)."""
    sink = torch.zeros(64, dtype=torch.float32, device=dev)
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev)     # 1 GiB
    dst = torch.empty_like(src)
    wgs, iters = 2048, 4096

    def timed(fn):
        fn()
        ms = []
        for _ in range(5):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            b.synchronize()
            ms.append(a.elapsed_time(b))
        return sorted(ms)[2]
    t_mfma = timed(lambda: tofu.probe_mfma(sink, iters, wgs))
    t_copy = timed(lambda: tofu.probe_copy(dst, src))
    return {"mfma_loop_tflops": round(wgs * 4 * iters * 8 * 4096 / t_mfma * 1e-9, 1),
            "copy_1gib_gbs": round(2 * src.numel() * 4 / t_copy * 1e-6, 1)}


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
    which = [s for s in args.legs.split(",") if s] or None
    names = which if which else list(tofu_workloads.STEP_LEGS) + list(tofu_workloads.EXTRA_LEGS)
    built = tofu_workloads.build(dev, names, keep_host=not args.no_cpu_baseline)
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
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(legs) + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(ev[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_per_step = wall * 1e3 / args.steps
    per_step = [[ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(args.steps)] for i in range(len(legs))]
    leg_ms = [sum(t) / len(t) for t in per_step]
    leg_out = []
    for leg, ms, samples in zip(legs, leg_ms, per_step):
        peak, unit = PEAK[leg.bound]
        scale = 1e-9 if leg.bound == "mfma" else 1e-6           # FLOP/ms -> TFLOP/s, B/ms -> GB/s
        achieved = leg.work / ms * scale
        # ms = mean over the timed steps (what `value` is made of); median and min over the same launches.
        # Inside a step every leg finds its operands evicted by the other legs (a step moves about 3 GB): cache-cold.
        entry = {"leg": leg.name, "bound": leg.bound, "ms": round(ms, 4), "median_ms": round(sorted(samples)[len(samples) // 2], 4),
                 "min_ms": round(min(samples), 4), "achieved": round(achieved, 2), "unit": unit, "frac": round(achieved / peak, 4)}
        if leg.conventional_flop:
            entry["conventional_tflops"] = round(leg.conventional_flop / ms * 1e-9, 2)
        leg_out.append(entry)
    flop = sum(l.work for l in legs if l.bound == "mfma")
    # the roofline object repeats the contraction leg that takes longest (its fix-up kernel included)
    dom = max([e for e in leg_out if e["bound"] == "mfma"] or leg_out, key=lambda e: e["ms"])
    traffic = None
    if dom["leg"] in TRAFFIC_KIB:
        traffic = round(1024.0 * sum(k * f for k, f in zip(TRAFFIC_KIB[dom["leg"]], TRAFFIC_SCALE)))
    out = {
        "metric": METRIC, "value": round(flop / (ms_per_step * 1e-3) * 1e-12, 3), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "one step = every leg of the shard path at full size: " + ", ".join(l.name for l in legs),
                   "shapes": "LSTM gate GEMM 128x32768x16384 (8-way N and K shards); 3x3 conv 2560ch 14x14 batch 128 "
                             "(C_out/8 and C_out/8 x H/2 shards, halo fetch); 3x3 wgrad 1280ch 28x28 (batch/8 shard); 8-way reduces"},
        "roofline": {"kernel": dom["leg"] + ": " + LEG_KERNELS.get(dom["leg"], ""), "bound": dom["bound"], "achieved": dom["achieved"], "peak": PEAK[dom["bound"]][0],
                     "unit": dom["unit"], "frac": dom["frac"], "traffic": traffic},
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
    # the streaming legs again, launched back to back: their operands are then partly resident in the
    # last-level cache (the gate reduce's 151 MB fit it, the dW reduce's 531 MB do not) -- the cache-warm figure
    for leg, entry in zip(legs, leg_out):
        if leg.bound != "hbm":
            continue
        for _ in range(3):
            leg.run()
        e = [torch.cuda.Event(enable_timing=True) for _ in range(21)]
        for i in range(20):
            e[i].record()
            leg.run()
        e[20].record()
        torch.cuda.synchronize()
        warm = sorted(e[i].elapsed_time(e[i + 1]) for i in range(20))[10]
        entry["back_to_back_ms"] = round(warm, 4)
        entry["back_to_back_gbs"] = round(leg.work / warm * 1e-6, 1)
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
        out["cpu_baseline"] = cpu_baseline(legs)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
