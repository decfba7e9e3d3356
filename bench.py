#!/usr/bin/env python3
"""Benchmark of the EXEC hot path on one MI355X.

A step is one EXEC of ResNet-50 (224x224, fp16 storage, fp32 accumulation) at
batch 16 over a synthetic batch that is already resident in HBM (INPUT done once
before the timed region): input cast, stem, max pool, 52 convolutions, global
average pool, FC and softmax, all through the C ABI.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-extra-configs]

Besides the headline line it measures, in the same run:
  * the EXEC latency profile of every batch size 1..16 over seeded images (on-device
    duration of --profile-repeats EXECs each: p50, p99, p99.9, p99.99, max) and the host
    wall time enqueue -> sync next to it;
  * every launch of the batch-16 plan, issued once each in plan order between its own
    pair of HIP events on the EXEC stream, many repetitions: the convolution kernel's
    achieved TFLOP/s against the dense fp16 MFMA peak, and against the per-launch
    composite roof max(t_MFMA, t_HBM);
  * workload configurations 3 (EXEC under a concurrent LOAD) and 4 (ResNet-152 bf16);
  * the CPU oracle on the host cores, as a reported baseline.
"""
import argparse
import json
import os
import re
import sys
import time
import types

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F16_TFLOPS = 2500.0   # MI355X dense fp16/bf16 MFMA
PEAK_HBM_GBS = 8000.0
BATCHES = (1, 2, 4, 8, 16)
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "exec_resnet50_b16_hbm_traffic.txt")


def counter_traffic_bytes():
    """HBM-side bytes of the convolution launches of one batch-16 EXEC, from the committed summary
    of the FETCH_SIZE / WRITE_SIZE counter runs (counters cannot be read from inside this process).
    None when the summary is missing or has no such line."""
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return None
    m = re.search(r"conv launches:\s+read ([\d.]+) MB \+ written ([\d.]+) MB", text)
    return (float(m.group(1)) + float(m.group(2))) * 1e6 if m else None


def cpu_baseline(seed, log):
    """The oracle as it stands, one image per host thread, on a bounded sample."""
    from oracle import network as N
    from oracle import topology as T
    from workload import gen
    cores = len(os.sched_getaffinity(0))
    threads = min(cores, 16)
    ops = T.resnet(50)
    w, b = gen.model_tensors(T.weight_shapes(ops), seed)
    n = 3 * threads   # about 15 s of host work
    x = gen.images(seed, 0, n, 3, 224, 224, "normal")
    t0 = time.perf_counter()
    N.forward(ops, w, b, x, threads=threads)
    dt = time.perf_counter() - t0
    log("cpu_baseline: %d images on %d threads in %.1f s" % (n, threads, dt))
    return {"value": n / dt, "unit": "inferences/s", "cores": threads, "kind": "oracle",
            "sample": "ResNet-50 224x224 fp32 nested-loop oracle, %d images of the same seeded workload, "
                      "one image at a time per thread, %.1f s wall" % (n, dt)}


def nearest_rank(v, q):
    import numpy as np
    s = np.sort(np.asarray(v, dtype=np.float64))
    k = min(len(s), max(1, int(np.ceil(q * len(s)))))
    return float(s[k - 1])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--profile-repeats", type=int, default=10000)
    ap.add_argument("--launch-reps", type=int, default=200, help="repetitions of the per-launch pass")
    ap.add_argument("--batch", type=int, default=16)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-configs", action="store_true", help="skip workload configurations 3 and 4")
    ap.add_argument("--layers-out", default="", help="write the per-launch table here (text)")
    ap.add_argument("--timed-only", action="store_true",
                    help="profiling runs: only the timed EXECs and the per-launch pass at --batch "
                         "(no per-batch latency profile, no extra configurations, no CPU baseline)")
    ap.add_argument("--no-graphs", action="store_true", help="issue every kernel as its own launch")
    ap.add_argument("--panels", action="store_true",
                    help="plan the tile numbering in channel panels (cw_set_panels; for the traffic counter runs)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="also run one device-to-device copy kernel of this many MiB (scale for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (an 8-GPU node is 8 independent workers); "
                 "run with --gpus 1")

    def log(msg):
        print("[bench] " + msg, file=sys.stderr, flush=True)

    import numpy as np
    import torch

    from paper_2006_02464_amd.runner import Worker, pinned_like
    from workload import gen

    seed = 0
    wk = Worker(workspace_bytes=512 << 20, io_bytes=512 << 20, weight_pool_bytes=1 << 30,
                load_staging_bytes=256 << 20)
    ctx, stream = wk.ctx, wk.stream
    if args.no_graphs:
        ctx.set_use_graphs(0)
    if args.copy_calibration:
        # a plain elementwise copy: reads and writes exactly this many bytes each
        src = torch.ones(args.copy_calibration << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.panels:
        ctx.set_panels(1)
    mid = ctx.model_define_resnet(50, 224, 224, "fp16")
    ops = ctx.model_get_ops(mid)
    shapes = [(o[2], o[1], o[3], o[4]) if o[0] == 0 else (o[2], o[1], 1, 1) for o in ops if o[0] in (0, 3)]
    w, b = gen.model_tensors(shapes, seed, "fp16")
    wk.load(mid, gen.pack_blob(w, b, "fp16"))
    del w, b
    B = args.batch
    images = gen.images(seed, 0, 16, 3, 224, 224, "normal", "fp16")
    x = pinned_like(images[:B])
    slot = ctx.input(mid, B, x, stream)
    stream.synchronize()
    log("model loaded, input resident")

    # ---- timed region: K EXECs back to back on one stream
    for _ in range(args.warmup):
        ctx.exec(mid, B, slot, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ctx.exec(mid, B, slot, stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = B * args.steps / dt
    log("batch %d: %.1f us/step wall, %.0f inferences/s" % (B, ms_per_step * 1e3, value))

    # ---- every launch of the plan, in plan order, one issue each between its own pair of HIP
    # events on the EXEC stream (a separate pass: event pairs inside the timed region would perturb
    # it).  An event pair adds the same dispatch-and-marker overhead to every launch; it is fixed by
    # requiring the launches to add up to the on-device duration of whole EXECs issued the same way
    # (plain launches, one event pair around the EXEC), and taken off every launch.
    plan = ctx.plan(mid, B)
    ctx.set_use_graphs(0)
    for _ in range(20):
        ctx.exec(mid, B, slot, stream)
    whole = []
    for _ in range(max(50, args.launch_reps)):
        ctx.exec(mid, B, slot, stream)
        whole.append(ctx.exec_duration_ns(slot) / 1e3)
    t_exec_plain = float(np.median(whole))
    ctx.exec_timed_launches(mid, B, slot, stream, inner=1)
    passes = np.stack([ctx.exec_timed_launches(mid, B, slot, stream, inner=1) for _ in range(args.launch_reps)])
    if not args.no_graphs:
        ctx.set_use_graphs(1)
    raw = np.median(passes, axis=0)
    overhead = (float(raw.sum()) - t_exec_plain) / len(plan)
    per = raw - overhead
    conv = [i for i, l in enumerate(plan) if l["kind"] == 1]
    conv_us = float(sum(per[i] for i in conv))
    conv_flops = float(sum(plan[i]["flops"] for i in conv))
    conv_bytes = float(sum(plan[i]["bytes"] for i in conv))
    achieved = conv_flops / (conv_us * 1e-6) / 1e12
    roof_us = [max(l["flops"] / (PEAK_MFMA_F16_TFLOPS * 1e6), l["bytes"] / (PEAK_HBM_GBS * 1e3)) for l in plan]
    conv_roof_us = float(sum(roof_us[i] for i in conv))
    lines = ["%-22s %4s %9s %6s %5s %7s %10s %9s %8s %8s %7s %8s" % (
        "launch", "op", "M", "N", "K", "grid", "GFLOP", "MB", "us", "TFLOP/s", "GB/s", "roof us")]
    for l, us, r in zip(plan, per, roof_us):
        lines.append("%-22s %4d %9d %6d %5d %7d %10.3f %9.2f %8.2f %8.1f %7.0f %8.2f" % (
            l["name"], l["op_index"], l["gemm_m"], l["gemm_n"], l["gemm_k"], l["grid_x"] * l["grid_y"],
            l["flops"] / 1e9, l["bytes"] / 1e6, us, l["flops"] / (us * 1e-6) / 1e12, l["bytes"] / (us * 1e-6) / 1e9, r))
    lines.append("whole EXEC (plain launches) %.1f us on-device; event overhead taken off every launch %.2f us; "
                 "conv launches %d, %.1f us; composite roof of the conv launches %.1f us" % (
                     t_exec_plain, overhead, len(conv), conv_us, conv_roof_us))
    if args.layers_out:
        with open(args.layers_out, "w") as f:
            f.write("\n".join(lines) + "\n")
    log("conv kernel: %d launches, %.1f us of a %.1f us EXEC, %.1f TFLOP/s, %.0f GB/s algorithmic; event overhead %.2f us per launch" % (
        len(conv), conv_us, t_exec_plain, achieved, conv_bytes / (conv_us * 1e-6) / 1e9, overhead))

    # ---- EXEC latency profile per batch size over seeded images: on-device durations, and the
    # host wall time enqueue -> sync of single EXECs next to them
    latency = {}
    for bs in (() if args.timed_only else BATCHES):
        s_b = ctx.input(mid, bs, pinned_like(images[:bs]), stream)
        stream.synchronize()
        ctx.profile_measure(mid, bs, 100, slot=s_b)
        p = ctx.profile_measure(mid, bs, args.profile_repeats, slot=s_b)
        wall = []
        for _ in range(300):
            t1 = time.perf_counter()
            ctx.exec(mid, bs, s_b, stream)
            stream.synchronize()
            wall.append((time.perf_counter() - t1) * 1e6)
        ctx.release(s_b)
        latency[str(bs)] = {"p50_us": round(p["p50_us"], 2), "p99_us": round(p["p99_us"], 2),
                            "p999_us": round(p["p999_us"], 2), "p9999_us": round(p["p9999_us"], 2),
                            "min_us": round(p["min_us"], 2), "max_us": round(p["max_us"], 2), "n": p["n"],
                            "inferences_per_s": round(bs / (p["p50_us"] * 1e-6), 1),
                            "p999_over_p50": round(p["p999_us"] / p["p50_us"], 4),
                            "p9999_over_p50": round(p["p9999_us"] / p["p50_us"], 4),
                            "host_wall_p50_us": round(nearest_rank(wall, 0.5), 2),
                            "host_wall_p99_us": round(nearest_rank(wall, 0.99), 2)}
        log("batch %2d: on-device p50 %.1f us p99 %.1f p99.9 %.1f p99.99 %.1f max %.1f; host wall p50 %.1f us" % (
            bs, p["p50_us"], p["p99_us"], p["p999_us"], p["p9999_us"], p["max_us"], latency[str(bs)]["host_wall_p50_us"]))
    ctx.release(slot)
    wk.close()

    traffic = counter_traffic_bytes() if B == 16 else None
    out = {
        "metric": "ResNet-50 inferences/s and exec p50/p99.9 latency at batch 1-16",
        "value": round(value, 1), "unit": "inferences/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "ResNet-50 224x224x3, fp16 He-normal weights, folded-BN bias, N(0,1) inputs, "
                               "EXEC at batch %d, input resident in HBM" % B,
                   "batch": B, "global_batch": B, "parallelism": "single GPU"},
        "exec_latency_us": latency,
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_MFMA_F16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / PEAK_MFMA_F16_TFLOPS, 4),
                     "traffic": traffic,
                     "traffic_unit": "bytes per EXEC over the conv launches (FETCH_SIZE + WRITE_SIZE counter runs, "
                                     "profiles/exec_resnet50_b16_hbm_traffic.txt)",
                     "algorithmic_bytes": conv_bytes,
                     "kernel": "conv_dlds_kernel (all %d convolution launches of one EXEC)" % len(conv),
                     "launches": len(conv), "conv_us_per_exec": round(conv_us, 2),
                     "avg_launch_us": round(conv_us / len(conv), 3),
                     "algorithmic_GBps": round(conv_bytes / (conv_us * 1e-6) / 1e9, 1),
                     "composite_roof_us": round(conv_roof_us, 2),
                     "composite_frac": round(conv_roof_us / conv_us, 4),
                     "exec_us_plain_launches": round(t_exec_plain, 2),
                     "exec_composite_frac": round(float(sum(roof_us)) / t_exec_plain, 4),
                     "event_overhead_us_per_launch": round(overhead, 3)},
    }
    if not args.timed_only and not args.no_extra_configs:
        from paper_2006_02464_amd import measure
        margs = types.SimpleNamespace(execs=2000, loads_per_round=6)
        for name, fn in (("config3_exec_under_concurrent_load", measure.config3), ("config4_resnet152_bf16_b16", measure.config4)):
            t1 = time.perf_counter()
            out[name] = fn(margs, log)
            log("%s: %.1f s" % (name, time.perf_counter() - t1))
    if not args.no_cpu_baseline and not args.timed_only:
        out["cpu_baseline"] = cpu_baseline(seed, log)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
