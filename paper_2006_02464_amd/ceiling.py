"""What the convolution kernel reaches on a compute-bound shape, per tile variant (needs an MI355X).

ResNet-50's own layers at batch <= 16 are small (49 to 392 tiles of 128x128) or HBM-bound, so their
TFLOP/s mix the quality of the kernel's inner loop with the shape's wave quantisation and fixed
costs.  This separates the two: through the C ABI it defines a model whose second operator is one
large convolution,

  gemm: 1x1, 2048 -> 2048 channels over 56x56 pixels at batch 16   (M 50176 x N 2048 x K 2048, 421 GFLOP)
  conv: 3x3,  512 ->  512 channels over 56x56 pixels at batch 16   (M 50176 x N  512 x K 4608, 237 GFLOP)

forces one tile variant after the other on it (cw_set_plan_override) and times that launch with HIP
events on the EXEC stream (cw_exec_timed_launches).  Prints a table; --out writes it to a file.

  python -m paper_2006_02464_amd.ceiling [--out FILE] [--tiles 128x128,128x64k128,...]
"""
import argparse
import sys

import numpy as np

CASES = {
    "gemm": dict(c=2048, k=1, pad=0),
    "conv": dict(c=512, k=3, pad=1),
}
HW, B = 56, 16


def ops_for(c, k, pad):
    # (op, cin, cout, kh, kw, stride, pad, relu, residual_from, input_from)
    return [(0, 3, c, 1, 1, 1, 0, 1, -1, -1),
            (0, c, c, k, k, 1, pad, 1, -1, 0),
            (2, c, c, 0, 0, 1, 0, 0, -1, 1),
            (3, c, 256, 1, 1, 1, 0, 0, -1, 2),
            (4, 256, 256, 0, 0, 1, 0, 0, -1, 3)]


def main():
    from .binding import CONV_TILES
    from .runner import Worker, pinned_like
    from workload import gen
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default="")
    ap.add_argument("--tiles", default="")
    ap.add_argument("--reps", type=int, default=7)
    args = ap.parse_args()
    tiles = args.tiles.split(",") if args.tiles else list(CONV_TILES)
    wk = Worker(workspace_bytes=2 << 30, io_bytes=64 << 20, weight_pool_bytes=256 << 20, load_staging_bytes=64 << 20)
    ctx = wk.ctx
    lines = ["%-6s %-14s %6s %9s %10s %9s" % ("case", "tile", "grid", "us", "TFLOP/s", "of 2500")]
    for name, cs in CASES.items():
        ops = ops_for(**cs)
        shapes = [(o[2], o[1], o[3], o[4]) if o[0] == 0 else (o[2], o[1], 1, 1) for o in ops if o[0] in (0, 3)]
        w, b = gen.model_tensors(shapes, 0, "fp16")
        blob = pinned_like(gen.pack_blob(w, b, "fp16"))
        x = pinned_like(gen.images(0, 0, B, 3, HW, HW, "normal", "fp16"))
        for tile in tiles:
            ctx.set_plan_override(tile, 1)
            try:
                mid = ctx.model_define(ops, 3, HW, HW, batch_sizes=(B,))
            finally:
                ctx.set_plan_override(-1, 0)
            ctx.load_weights(mid, blob, wk.stream)
            slot = ctx.input(mid, B, x, wk.stream)
            plan = ctx.plan(mid, B)
            idx = [i for i, l in enumerate(plan) if l["op_index"] == 1 and l["kind"] == 1][0]
            ctx.exec_timed_launches(mid, B, slot, wk.stream, inner=1)
            us = float(np.median([ctx.exec_timed_launches(mid, B, slot, wk.stream, inner=3)[idx] for _ in range(args.reps)]))
            l = plan[idx]
            tf = l["flops"] / (us * 1e-6) / 1e12
            lines.append("%-6s %-14s %6d %9.1f %10.1f %9.3f" % (name, tile,
                                                                l["grid_x"] * l["grid_y"], us, tf, tf / 2500.0))
            print(lines[-1], file=sys.stderr, flush=True)
            ctx.release(slot)
            ctx.unload_weights(mid)
    wk.close()
    text = "\n".join(lines)
    print(text)
    if args.out:
        with open(args.out, "w") as f:
            f.write(text + "\n")


if __name__ == "__main__":
    sys.exit(main())
