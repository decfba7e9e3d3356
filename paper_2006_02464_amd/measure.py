"""Measurements beyond bench.py's headline line, one per workload configuration (needs an MI355X).

  python -m paper_2006_02464_amd.measure --config 3   EXEC latency with and without a concurrent LOAD
  python -m paper_2006_02464_amd.measure --config 4   ResNet-152, bf16, batch 16: throughput and latency
  python -m paper_2006_02464_amd.measure --config 5   64 resident ResNet-50s, Poisson arrivals, mixed batch sizes
  python -m paper_2006_02464_amd.measure --config 6   INFER actions with earliest/latest through the worker's executors
  python -m paper_2006_02464_amd.measure --config 8   ResNet-50 EXEC under each plan option (fusion, pair launches, graphs,
                                                      Winograd, resident multi-layer launch) against the default plan
  python -m paper_2006_02464_amd.measure --config 7   the other Table-1 families (MobileNet-, DenseNet-, Inception-style
                                                      operator lists): EXEC latency and every launch against its roofline

Each prints one JSON object.  All inputs are synthetic (seeded, workload/gen.py); EXEC time depends
on the values only through power and clocks (a few percent), so every profile is taken over seeded images.  Durations are on-device (the event pair around every EXEC); the host thread
issues INPUT / EXEC / OUTPUT as the worker of the paper does: copies on one stream, EXEC on another,
one EXEC at a time.
"""
import argparse
import json
import sys
import time

import numpy as np


def pct(v, q):
    """Nearest-rank percentile of a sample."""
    s = np.sort(np.asarray(v, dtype=np.float64))
    k = min(len(s), max(1, int(np.ceil(q * len(s)))))
    return float(s[k - 1])


def summary(v):
    return {"n": len(v), "p50_us": round(pct(v, 0.5), 2), "p99_us": round(pct(v, 0.99), 2),
            "p999_us": round(pct(v, 0.999), 2), "max_us": round(float(np.max(v)), 2),
            "p999_over_p50": round(pct(v, 0.999) / pct(v, 0.5), 4)}


def resnet_blob(ctx, mid, seed, dtype):
    from workload import gen
    ops = ctx.model_get_ops(mid)
    # (cout, cin per group, kh, kw) per convolution, (out, in, 1, 1) per FC
    shapes = [(o[2], o[1] // max(1, o[11]), o[3], o[4]) if o[0] == 0 else (o[2], o[1], 1, 1) for o in ops if o[0] in (0, 3)]
    w, b = gen.model_tensors(shapes, seed, dtype)
    return gen.pack_blob(w, b, dtype)


def exec_rounds(ctx, mid, batch, slots, stream, rounds, between=None):
    """`rounds` x len(slots) back-to-back EXECs; returns every on-device duration in us."""
    out = []
    for r in range(rounds):
        for s in slots:
            ctx.exec(mid, batch, s, stream)
        if between is not None:
            between(r)
        out.extend(ctx.exec_duration_ns(s) / 1e3 for s in slots)   # blocks until each has finished
    return out


def config3(args, log):
    import torch
    from .runner import Worker, pinned_like
    from workload import gen
    B, n_slots = 8, 20
    wk = Worker(workspace_bytes=512 << 20, io_bytes=512 << 20, weight_pool_bytes=1 << 30, load_staging_bytes=256 << 20)
    ctx, ex = wk.ctx, wk.stream
    ld = torch.cuda.Stream()
    m1 = ctx.model_define_resnet(50, 224, 224, "fp16")
    m2 = ctx.model_define(ctx.model_get_ops(m1), 3, 224, 224, batch_sizes=(B,))
    blob1 = pinned_like(resnet_blob(ctx, m1, 0, "fp16"))
    blob2 = pinned_like(resnet_blob(ctx, m2, 1, "fp16"))
    ctx.load_weights(m1, blob1, ex)
    x = pinned_like(gen.images(0, 0, B, 3, 224, 224, "normal", "fp16"))
    slots = [ctx.input(m1, B, x, ex) for _ in range(n_slots)]
    ex.synchronize()
    exec_rounds(ctx, m1, B, slots, ex, 5)                                  # warm-up
    alone = exec_rounds(ctx, m1, B, slots, ex, args.execs // n_slots)
    loads = [0]

    def reload(_):
        # keep LOADs (51 MB host-to-device copy + weight packing each) queued on their own stream
        for _k in range(args.loads_per_round):
            ctx.unload_weights(m2)
            ctx.load_weights(m2, blob2, ld)
            loads[0] += 1

    # device time of one LOAD on an otherwise idle GPU
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ctx.load_weights(m2, blob2, ld)
    ld.synchronize()
    ctx.unload_weights(m2)
    e0.record(ld)
    ctx.load_weights(m2, blob2, ld)
    e1.record(ld)
    ld.synchronize()
    load_ms = e0.elapsed_time(e1)
    t0 = time.perf_counter()
    under = exec_rounds(ctx, m1, B, slots, ex, args.execs // n_slots, between=reload)
    ld.synchronize()
    dt = time.perf_counter() - t0
    wk.close()
    return {"config": 3, "workload": "ResNet-50 fp16 batch 8, %d back-to-back EXECs; second ResNet-50 (51 MB) "
                                     "unloaded and re-LOADed from pinned memory on another stream throughout" % len(under),
            "exec_alone": summary(alone), "exec_under_load": summary(under),
            "p50_ratio": round(pct(under, 0.5) / pct(alone, 0.5), 4),
            "loads_completed": loads[0], "one_load_ms_idle_gpu": round(load_ms, 3),
            "load_busy_fraction_of_wall": round(min(1.0, loads[0] * load_ms * 1e-3 / dt), 3), "wall_s": round(dt, 3)}


def config4(args, log):
    import torch
    from .runner import Worker, pinned_like
    from workload import gen
    B = 16
    wk = Worker(workspace_bytes=512 << 20, io_bytes=256 << 20, weight_pool_bytes=1 << 30, load_staging_bytes=512 << 20)
    ctx, ex = wk.ctx, wk.stream
    mid = ctx.model_define_resnet(152, 224, 224, "bf16")
    ctx.load_weights(mid, pinned_like(resnet_blob(ctx, mid, 0, "bf16")), ex)
    x = pinned_like(gen.images(0, 0, B, 3, 224, 224, "normal", "bf16"))
    slot = ctx.input(mid, B, x, ex)
    ex.synchronize()
    for _ in range(50):
        ctx.exec(mid, B, slot, ex)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.execs):
        ctx.exec(mid, B, slot, ex)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = ctx.profile_measure(mid, B, 1000, slot=slot)
    plan = ctx.plan(mid, B)
    wk.close()
    return {"config": 4, "workload": "ResNet-152 224x224 bf16 storage (fp16 overflows with these weights), batch 16",
            "inferences_per_s": round(B * args.execs / dt, 1), "ms_per_exec_wall": round(dt / args.execs * 1e3, 4),
            "exec": {k: round(prof[k], 2) for k in ("p50_us", "p99_us", "p999_us", "min_us", "max_us")},
            "launches": len(plan), "gflop_per_exec": round(sum(l["flops"] for l in plan) / 1e9, 1),
            "tflops": round(sum(l["flops"] for l in plan) / (prof["p50_us"] * 1e-6) / 1e12, 1)}


def config5(args, log):
    import torch
    from .runner import Worker, pinned_like
    from workload import gen
    n_models, batches = 64, (1, 2, 4, 8, 16)
    wk = Worker(workspace_bytes=512 << 20, io_bytes=1 << 30, weight_pool_bytes=4 << 30, load_staging_bytes=256 << 20)
    ctx, ex = wk.ctx, wk.stream
    cp = torch.cuda.Stream()
    mids = [ctx.model_define_resnet(50, 224, 224, "fp16") for _ in range(n_models)]
    # 64 independently seeded weight sets (seeds 0..63), drawn on a few host threads
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=8) as pool:
        blobs = list(pool.map(lambda s: resnet_blob(ctx, mids[0], s, "fp16"), range(n_models)))
    for k, m in enumerate(mids):
        staged = pinned_like(blobs[k])
        ctx.load_weights(m, staged, ex)
        ex.synchronize()
        blobs[k] = None
    log("64 models resident, %.2f GB of the weight pool in use" % (((4 << 30) - ctx.weight_pool_free()) / 1e9))
    xs = {b: pinned_like(gen.images(0, 0, b, 3, 224, 224, "normal", "fp16")) for b in batches}
    probs = torch.empty((16, 1000), dtype=torch.float32, pin_memory=True)
    # capacity of the mix from the per-batch profile of one model
    p50 = {}
    for b in batches:
        s_b = ctx.input(mids[0], b, xs[b], ex)
        p50[b] = ctx.profile_measure(mids[0], b, 200, slot=s_b)["p50_us"]
        ctx.release(s_b)
    mean_exec_us = float(np.mean(list(p50.values())))
    lam = args.load / (mean_exec_us * 1e-6)                     # requests per second
    # seeded arrivals and request mix (counter-based generator of the workload module)
    n = args.requests
    u = gen.uniform01(args.seed, 1000, 3 * n)
    gaps = -np.log(1.0 - u[:n]) / lam
    arrive = np.cumsum(gaps)
    which = np.minimum((u[n:2 * n] * n_models).astype(int), n_models - 1)
    bsel = np.array(batches)[np.minimum((u[2 * n:] * len(batches)).astype(int), len(batches) - 1)]
    per_b = {b: [] for b in batches}
    inflight = []
    max_inflight = 24

    def drain_one():
        slot, b = inflight.pop(0)
        per_b[b].append(ctx.exec_duration_ns(slot) / 1e3)
        ctx.output(slot, probs[:b], None, cp)

    late = 0.0
    t0 = time.perf_counter()
    for i in range(n):
        while time.perf_counter() - t0 < arrive[i]:
            pass
        late = max(late, time.perf_counter() - t0 - arrive[i])
        b, m = int(bsel[i]), mids[int(which[i])]
        slot = ctx.input(m, b, xs[b], cp)
        ctx.exec(m, b, slot, ex)
        inflight.append((slot, b))
        if len(inflight) >= max_inflight:
            drain_one()
    while inflight:
        drain_one()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    wk.close()
    images = int(bsel.sum())
    return {"config": 5, "workload": "%d ResNet-50 fp16 weight sets resident (independently seeded, seeds 0..%d), "
                                     "%d requests, Poisson arrivals at %.0f req/s = %.2f x capacity of "
                                     "the mix, model ~U{0..63}, batch ~U{1,2,4,8,16}, seed %d"
                                     % (n_models, n_models - 1, n, lam, args.load, args.seed),
            "inferences_per_s": round(images / wall, 1), "requests_per_s": round(n / wall, 1), "wall_s": round(wall, 3),
            "max_host_lateness_ms": round(late * 1e3, 3),
            "single_model_p50_us": {str(b): round(p50[b], 2) for b in batches},
            "exec_by_batch": {str(b): summary(per_b[b]) for b in batches}}


def config6(args, log):
    """A schedule of INFER actions as a controller would send it (paper sections 4.4, 5.2): one ResNet-50,
    batch 16, action i may begin at t0 + i * period with period = 1.15 x the measured EXEC p50 and must
    have begun 1 ms later.  Beside them a second ResNet-50 is unloaded and loaded again every 100 INFERs
    (the controller's LOAD / UNLOAD actions, which section 5.2 runs next to EXEC).  Reports how
    punctually EXEC begins (all actions, and those whose window overlaps a LOAD), what the executors
    add around the on-device time, how long a LOAD occupies its executor, and how many actions the
    window rejected."""
    import torch
    from .binding import CW_ACTION_INFER, CW_ACTION_LOAD, CW_ACTION_UNLOAD, Executors
    from .runner import Worker, pinned_like
    from workload import gen
    B, n = 16, args.requests if args.requests != 10000 else 2000
    every = 100
    wk = Worker(workspace_bytes=512 << 20, io_bytes=512 << 20, weight_pool_bytes=1 << 30, load_staging_bytes=256 << 20)
    ctx = wk.ctx
    mid = ctx.model_define_resnet(50, 224, 224, "fp16")
    blob = pinned_like(resnet_blob(ctx, mid, 0, "fp16"))
    ctx.load_weights(mid, blob, wk.stream)
    wk.stream.synchronize()
    x = pinned_like(gen.images(0, 0, B, 3, 224, 224, "normal", "fp16"))
    s_p = ctx.input(mid, B, x, wk.stream)
    p50 = ctx.profile_measure(mid, B, 300, slot=s_p)["p50_us"]
    ctx.release(s_p)
    ctx.unload_weights(mid)
    other = ctx.model_define_resnet(50, 224, 224, "fp16")
    blob2 = pinned_like(resnet_blob(ctx, other, 1, "fp16"))
    # How long the LOAD call itself keeps the context (it only enqueues the copies and pack kernels
    # and records the plans' graphs; the executors issue nothing else meanwhile): first LOAD, LOAD
    # into the same pages again, LOAD into other pages.
    import time
    call_ms = []
    for k in range(3):
        if k == 2:
            ctx.load_weights(mid, blob, wk.stream)           # takes the lowest pages, so `other` lands elsewhere
        t_a = time.perf_counter()
        ctx.load_weights(other, blob2, wk.stream)
        call_ms.append(round((time.perf_counter() - t_a) * 1e3, 3))
        wk.stream.synchronize()
        ctx.unload_weights(other)
    ctx.unload_weights(mid)
    ex = Executors(ctx)
    probs = [torch.empty((B, 1000), dtype=torch.float32, pin_memory=True) for _ in range(32)]
    now = ex.now_ns()
    ex.submit(-1, CW_ACTION_LOAD, mid, now, now + 10**9, host_in=blob)
    load = ex.next_result(10.0)
    period = int(p50 * 1.15 * 1e3)
    t0 = ex.now_ns() + 20_000_000
    res, loads, unloads, sent, side, side_out = [], [], [], 0, 0, 0
    LOAD_ID, UNLOAD_ID = 1 << 20, 1 << 21
    while len(res) < n or side_out:
        while sent < n and sent - len(res) < 24:                 # a controller keeps a short queue ahead
            if sent % every == every // 2:                        # the other model goes out and comes back in
                at = t0 + sent * period
                if side:
                    ex.submit(UNLOAD_ID + side, CW_ACTION_UNLOAD, other, at, at + 50_000_000)
                    side_out += 1
                ex.submit(LOAD_ID + side, CW_ACTION_LOAD, other, at + (100_000 if side else 0), at + 50_000_000, host_in=blob2)
                side, side_out = side + 1, side_out + 1
            ex.submit(sent, CW_ACTION_INFER, mid, t0 + sent * period, t0 + sent * period + 1_000_000, batch=B, host_in=x,
                      host_probs=probs[sent % 32])
            sent += 1
        r = ex.next_result(10.0)
        assert r is not None
        if r["id"] >= UNLOAD_ID:
            unloads.append(r); side_out -= 1
        elif r["id"] >= LOAD_ID:
            loads.append(r); side_out -= 1
        else:
            res.append(r)
    ex.destroy()
    wk.close()
    ok = [r for r in res if r["status"] == 0]
    late = [(r["begin_ns"] - (t0 + r["id"] * period)) / 1e3 for r in ok]
    spans = [(l["begin_ns"], l["end_ns"] + int(l["device_ns"])) for l in loads if l["status"] == 0]
    beside = [(r["begin_ns"] - (t0 + r["id"] * period)) / 1e3 for r in ok
              if any(a - period <= t0 + r["id"] * period <= b for a, b in spans)]
    dev_beside = [r["device_ns"] / 1e3 for r in ok if any(a - period <= t0 + r["id"] * period <= b for a, b in spans)]
    # the EXECs around the first three LOADs: (begin of EXEC minus begin of LOAD in us, on-device us)
    around = [[(round((r["begin_ns"] - a) / 1e3), round(r["device_ns"] / 1e3, 1)) for r in sorted(ok, key=lambda r: r["begin_ns"])
               if a - 2 * period <= r["begin_ns"] <= b + 2 * period] for a, b in spans[1:4]]
    over = [((r["end_ns"] - r["begin_ns"]) - r["device_ns"]) / 1e3 for r in ok]
    dev = [r["device_ns"] / 1e3 for r in ok]
    span = (max(r["end_ns"] for r in res) - t0) / 1e9
    return {"config": 6, "workload": "ResNet-50 fp16 batch 16: %d INFER actions through the executors, action i may begin at "
                                     "t0 + i x %.1f us (1.15 x EXEC p50 of %.1f us), window 1 ms" % (n, period / 1e3, p50),
            "load_action": {"status": load["status"], "host_ms": round((load["end_ns"] - load["begin_ns"]) / 1e6, 3), "device_ms": round(load["device_ns"] / 1e6, 3)},
            "load_call_host_ms": {"first": call_ms[0], "same_pages_again": call_ms[1], "other_pages": call_ms[2]},
            "side_actions": {"loads": len(loads), "loads_ok": sum(l["status"] == 0 for l in loads), "unloads_ok": sum(u["status"] == 0 for u in unloads),
                             "load_host_ms": {"p50": round(pct([(l["end_ns"] - l["begin_ns"]) / 1e6 for l in loads], 0.5), 3),
                                              "max": round(max((l["end_ns"] - l["begin_ns"]) / 1e6 for l in loads), 3)} if loads else None,
                             "load_device_ms": {"p50": round(pct([l["device_ns"] / 1e6 for l in loads], 0.5), 3),
                                                "max": round(max(l["device_ns"] / 1e6 for l in loads), 3)} if loads else None,
                             "infer_beside_a_load": len(beside),
                             "begin_after_earliest_us_beside_a_load": {"p50": round(pct(beside, 0.5), 1), "p99": round(pct(beside, 0.99), 1), "max": round(max(beside), 1)} if beside else None,
                             "exec_device_us_beside_a_load": summary(dev_beside) if dev_beside else None,
                             "execs_around_three_loads_offset_us_and_device_us": around},
            "executed": len(ok), "rejected_too_late": sum(r["status"] == -11 for r in res),
            "begin_after_earliest_us": {"p50": round(pct(late, 0.5), 1), "p99": round(pct(late, 0.99), 1), "max": round(max(late), 1)},
            "exec_device_us": summary(dev),
            "host_end_minus_begin_minus_device_us": {"p50": round(pct(over, 0.5), 1), "p99": round(pct(over, 0.99), 1)},
            "inferences_per_s": round(B * len(ok) / span, 1)}


# The operator lists of the other families, written out here for the library (the test suite holds
# its own copies on the oracle's side): (op, cin, cout, kh, kw, stride, pad, act, residual_from,
# input_from, pad_w, groups); op 0 conv, 1 max pool, 2 global average pool, 3 FC, 4 softmax, 5 concat.
def _tail(ops, cin, classes=1000):
    ops.append((2, cin, cin, 0, 0, 1, 0, 0, -1, len(ops) - 1, 0, 0))
    ops.append((3, cin, classes, 1, 1, 1, 0, 0, -1, len(ops) - 1, 0, 0))
    ops.append((4, classes, classes, 0, 0, 1, 0, 0, -1, len(ops) - 1, 0, 0))
    return ops


def mobilenet_ops():
    cfg = [(64, 1), (128, 2), (128, 1), (256, 2), (256, 1), (512, 2)] + [(512, 1)] * 5 + [(1024, 2), (1024, 1)]
    ops, cin = [(0, 3, 32, 3, 3, 2, 1, 1, -1, -1, 0, 0)], 32
    for i, (cout, stride) in enumerate(cfg):
        act, block_in = (2 if i >= 7 else 1), len(ops) - 1
        ops.append((0, cin, cin, 3, 3, stride, 1, act, -1, block_in, 0, cin))
        ops.append((0, cin, cout, 1, 1, 1, 0, act, block_in if (stride == 1 and cin == cout) else -1, len(ops) - 1, 0, 0))
        cin = cout
    return _tail(ops, cin)


def dense_ops(layers=(6, 12), growth=32, bottleneck=128, stem=64):
    ops = [(0, 3, stem, 7, 7, 2, 3, 1, -1, -1, 0, 0), (1, stem, stem, 3, 3, 2, 1, 0, -1, 0, 0, 0)]
    cin = stem
    for b, n in enumerate(layers):
        cur = len(ops) - 1
        for _ in range(n):
            ops.append((0, cin, bottleneck, 1, 1, 1, 0, 1, -1, cur, 0, 0))
            ops.append((0, bottleneck, growth, 3, 3, 1, 1, 1, -1, len(ops) - 1, 0, 0))
            ops.append((5, cin, cin + growth, 0, 0, 1, 0, 0, len(ops) - 1, cur, 0, 0))
            cur, cin = len(ops) - 1, cin + growth
        if b + 1 < len(layers):
            ops.append((0, cin, cin // 2, 1, 1, 1, 0, 1, -1, cur, 0, 0))
            cin //= 2
            ops.append((1, cin, cin, 2, 2, 2, 0, 0, -1, len(ops) - 1, 0, 0))
    return _tail(ops, cin)


def inception_ops(width=256, blocks=2):
    ops = [(0, 3, 32, 3, 3, 2, 1, 1, -1, -1, 0, 0), (0, 32, width, 3, 3, 2, 1, 1, -1, 0, 0, 0)]
    for _ in range(blocks):
        x = len(ops) - 1
        ops.append((0, width, width, 1, 1, 1, 0, 1, -1, x, 0, 0))
        a = len(ops) - 1
        ops.append((0, width, width, 1, 1, 1, 0, 1, -1, x, 0, 0))
        ops.append((0, width, width, 1, 7, 1, 0, 1, -1, len(ops) - 1, 3, 0))
        ops.append((0, width, width, 7, 1, 1, 3, 1, -1, len(ops) - 1, 0, 0))
        ops.append((5, width, 2 * width, 0, 0, 1, 0, 0, len(ops) - 1, a, 0, 0))
        ops.append((0, 2 * width, width, 1, 1, 1, 0, 1, x, len(ops) - 1, 0, 0))
    return _tail(ops, width)


def config7(args, log):
    """EXEC latency per batch size and the per-launch table at batch 16 of the three other families."""
    from .runner import Worker, pinned_like
    from workload import gen
    wk = Worker(workspace_bytes=1 << 30, io_bytes=256 << 20, weight_pool_bytes=512 << 20, load_staging_bytes=128 << 20)
    ctx, ex = wk.ctx, wk.stream
    out = {"config": 7, "families": {}}
    tables = []
    for name, ops, hw in (("mobilenet", mobilenet_ops(), 224), ("densenet-style", dense_ops(), 224), ("inception-style", inception_ops(), 224)):
        mid = ctx.model_define(ops, 3, hw, hw)
        shapes = [(o[2], o[1] // max(1, o[11]), o[3], o[4]) if o[0] == 0 else (o[2], o[1], 1, 1) for o in ops if o[0] in (0, 3)]
        w, b = gen.model_tensors(shapes, 0, "fp16")
        ctx.load_weights(mid, pinned_like(gen.pack_blob(w, b, "fp16")), ex)
        ex.synchronize()
        fam = {"params": int(sum(int(np.prod(s)) + s[0] for s in shapes)), "exec": {}}
        for B in (1, 4, 16):
            slot = ctx.input(mid, B, pinned_like(gen.images(0, 0, B, 3, hw, hw, "normal", "fp16")), ex)
            ctx.profile_measure(mid, B, 50, slot=slot)
            p = ctx.profile_measure(mid, B, 1000, slot=slot)
            fam["exec"][str(B)] = {"p50_us": round(p["p50_us"], 2), "p999_over_p50": round(p["p999_us"] / p["p50_us"], 4),
                                   "inferences_per_s": round(B / (p["p50_us"] * 1e-6), 1), "launches": ctx.plan_num_launches(mid, B)}
            if B == 16:
                plan = ctx.plan(mid, B)
                ctx.set_use_graphs(0)
                whole = []
                for _ in range(60):
                    ctx.exec(mid, B, slot, ex)
                    whole.append(ctx.exec_duration_ns(slot) / 1e3)
                raw = np.median(np.stack([ctx.exec_timed_launches(mid, B, slot, ex, inner=1) for _ in range(60)]), axis=0)
                ctx.set_use_graphs(1)
                over = (float(raw.sum()) - float(np.median(whole[10:]))) / len(plan)
                us = raw - over
                groups = {}
                for l, u in zip(plan, us):
                    key = l["name"].split("_s")[0] if l["name"].startswith(("dwconv", "conv")) else l["name"]
                    g = groups.setdefault(key, [0, 0.0, 0, 0])
                    g[0] += 1; g[1] += float(u); g[2] += l["bytes"]; g[3] += l["flops"]
                fam["by_kernel_b16"] = {k: {"launches": v[0], "us": round(v[1], 1), "GBps": round(v[2] / (v[1] * 1e-6) / 1e9, 0),
                                            "TFLOPs": round(v[3] / (v[1] * 1e-6) / 1e12, 1), "frac_of_8TBps": round(v[2] / (v[1] * 1e-6) / 8e12, 3)}
                                        for k, v in groups.items()}
                tables.append("== %s, %dx%d, batch 16: every launch (us net of %.2f us event overhead)" % (name, hw, hw, over))
                tables.append("%-26s %9s %6s %6s %8s %8s %8s %8s" % ("launch", "M", "N", "K", "MB", "us", "GB/s", "TFLOP/s"))
                for l, u in zip(plan, us):
                    tables.append("%-26s %9d %6d %6d %8.2f %8.2f %8.0f %8.1f" % (l["name"], l["gemm_m"], l["gemm_n"], l["gemm_k"], l["bytes"] / 1e6, u,
                                                                                   l["bytes"] / (u * 1e-6) / 1e9, l["flops"] / (u * 1e-6) / 1e12))
            ctx.release(slot)
        ctx.unload_weights(mid)
        out["families"][name] = fam
        log("%s: %s" % (name, fam["exec"]))
    wk.close()
    if args.table_out:
        with open(args.table_out, "w") as f:
            f.write("\n".join(tables) + "\n")
    return out


def config8(args, log):
    """The same ResNet-50, the same seeded images, one plan option changed at a time: launches per
    EXEC and the on-device EXEC p50 at batch 1 and 16 (1000 EXECs each), all in one process on one GPU."""
    from .runner import Worker, pinned_like
    from workload import gen
    wk = Worker(workspace_bytes=1 << 30, io_bytes=256 << 20, weight_pool_bytes=1 << 30, load_staging_bytes=256 << 20)
    ctx, ex = wk.ctx, wk.stream
    variants = [("default plan", None, None), ("fused 3x3+1x1 launches off", ctx.set_fusion, 1),
                ("next block's 1x1 reduce as a launch of its own", ctx.set_fusion_third, 1),
                ("max pool and the 1x1 behind it as two launches", ctx.set_fusion_pool, 1), ("pair launches off", ctx.set_pair_launches, 1),
                ("FC and softmax as one launch", ctx.set_fc_softmax, 0),
                ("tile numbering in channel panels where they move fewer bytes", ctx.set_panels, 0),
                ("plain launches instead of graph replay", None, None), ("Winograd F(2x2,3x3) for the 3x3 stride-1 layers", ctx.set_winograd, 0),
                ("resident multi-layer launches", ctx.set_resident, 0), ("resident launches for the later stages only", "resident2", 0), ("default plan again", None, None)]
    blob, rows = None, []
    for name, setter, default in variants:
        if setter == "resident2":
            ctx.set_resident(2)
            setter = ctx.set_resident
        elif setter is not None:
            setter(1 - default)
        try:
            mid = ctx.model_define_resnet(50, 224, 224, "fp16")
        finally:
            if setter is not None:
                setter(default)
        if blob is None:
            blob = pinned_like(resnet_blob(ctx, mid, 0, "fp16"))
        graphs = 0 if name.startswith("plain launches") else 1
        ctx.set_use_graphs(graphs)
        ctx.load_weights(mid, blob, ex)
        row = {"variant": name}
        for B in (1, 16):
            slot = ctx.input(mid, B, pinned_like(gen.images(0, 0, B, 3, 224, 224, "normal", "fp16")), ex)
            ctx.profile_measure(mid, B, 50, slot=slot)
            p = ctx.profile_measure(mid, B, 1000, slot=slot)
            row["b%d" % B] = {"launches": ctx.plan_num_launches(mid, B), "p50_us": round(p["p50_us"], 1), "p999_over_p50": round(p["p999_us"] / p["p50_us"], 4)}
            ctx.release(slot)
        ctx.set_use_graphs(1)
        ctx.unload_weights(mid)
        rows.append(row)
        log(str(row))
    wk.close()
    return {"config": 8, "workload": "ResNet-50 224x224 fp16, 1000 EXECs per cell", "variants": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True, choices=(3, 4, 5, 6, 7, 8))
    ap.add_argument("--table-out", default="", help="config 7: write the per-launch tables here")
    ap.add_argument("--execs", type=int, default=2000)
    ap.add_argument("--loads-per-round", type=int, default=6, help="config 3: LOADs queued per 20 EXECs")
    ap.add_argument("--requests", type=int, default=10000)
    ap.add_argument("--load", type=float, default=0.7, help="config 5: arrival rate as a fraction of capacity")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--graphs", type=int, default=-1, help="1 / 0: replay HIP graphs in EXEC or issue every launch (default: the library's)")
    args = ap.parse_args()

    def log(msg):
        print("[measure] " + msg, file=sys.stderr, flush=True)

    if args.graphs >= 0:   # applies to every context made below
        from . import runner
        make = runner.Worker.__init__

        def patched(self, **kw):
            make(self, **kw)
            self.ctx.set_use_graphs(args.graphs)
        runner.Worker.__init__ = patched
    out = {3: config3, 4: config4, 5: config5, 6: config6, 7: config7, 8: config8}[args.config](args, log)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    sys.exit(main())
