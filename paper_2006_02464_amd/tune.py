"""Offline tuning of the conv launch plan (a development tool; needs an MI355X).

For every batch size and every convolution GEMM shape of a ResNet this tries each
(tile, split-K) candidate *in place*: the candidate is installed for that one shape
with cw_set_plan_table, the model is defined and loaded, and the median on-device
duration of whole EXECs (the production path: HIP-graph replay, every other layer
as currently chosen, caches as warm or cold as they really are) decides.  One
pass of coordinate descent per batch size, starting from the library's current
choice.  The result is written as csrc/plan_table.inc, which the library compiles
in.  Nothing is tuned when EXEC runs.

  python -m paper_2006_02464_amd.tune [--family resnet] [--depth 50] [--hw 224] [--batches 1,2,4,8,16] [--out FILE] [--keep-existing]

The table as compiled in: ResNet-50 first, then `--depth 18 --keep-existing`, then the other
families' lists (`--family mobilenet|densenet|inception --batches 1,4,16 --keep-existing`), then a second
pass over each of those with `--protect-resnet 50` in place of `--keep-existing`.
"""
import argparse
import os
import re
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
TABLE = os.path.join(HERE, "csrc", "plan_table.inc")
SPLITS = (1, 2, 4, 8, 16)
TILE_DIMS = {"128x128": (128, 128), "128x64": (128, 64), "64x64": (64, 64), "64x32": (64, 32), "32x64": (32, 64),
             "32x32": (32, 32), "256x64": (256, 64), "128x128w8": (128, 128),
             "128x64k128": (128, 64), "64x64k128": (64, 64), "64x32k128": (64, 32), "32x64k128": (32, 64),
             "32x32k128": (32, 32),
             "128x64k128g2": (128, 64), "64x64k128g2": (64, 64), "64x64k128g4": (64, 64), "64x32k128g4": (64, 32),
             "32x64k128g4": (32, 64), "32x32k128g4": (32, 32),
             "32x32k128g8": (32, 32), "128x64g2": (128, 64), "64x64g2": (64, 64), "32x32g4": (32, 32)}
POOLS = dict(workspace_bytes=1024 << 20, io_bytes=64 << 20, weight_pool_bytes=512 << 20, load_staging_bytes=256 << 20)


def candidates(M, N, K, kh, stride=1):
    """(tile, split) pairs worth trying for one GEMM shape."""
    cin = K // (kh * kh)   # 3 for the first convolution: no k128 tiles, K slices are pairs of filter rows
    out = []
    for tile, (bm, bn) in TILE_DIMS.items():
        if bn > N or (bm > 64 and bm > M):
            continue
        if "k128" in tile and cin % 128 != 0:
            continue
        ktiles = K // (128 if "k128" in tile else 64)
        tiles = -(-M // bm) * -(-N // bn)
        for s in SPLITS:
            if s > 1 and (s > ktiles or tiles >= 1024 or M * N * 4 * s > (64 << 20)):
                continue
            out.append((tile, s))
    return out


def rows(table):
    return [k + v for k, v in table.items()]


def read_table(path):
    """{(M, N, K, kh, stride): (tile, split)} of a plan_table.inc."""
    out = {}
    for line in open(path):
        m = re.match(r"\{(\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+)\}", line)
        if m:
            v = tuple(int(g) for g in m.groups())
            out[v[:5]] = v[5:]
    return out


class Bench:
    def __init__(self, family, depth, hw, reps):
        from .runner import Worker, pinned_like
        from . import measure
        self.hw, self.reps = hw, reps
        self.wk = Worker(**POOLS)
        ctx = self.wk.ctx
        if family == "resnet":
            mid = ctx.model_define_resnet(depth, hw, hw)
        else:
            lists = {"mobilenet": measure.mobilenet_ops, "densenet": measure.dense_ops, "inception": measure.inception_ops}
            mid = ctx.model_define(lists[family](), 3, hw, hw, batch_sizes=(1,))
        self.ops = ctx.model_get_ops(mid)
        # seeded random weights, as every measurement uses: with all-zero operands the matrix cores draw
        # less power, the clocks sit higher and EXEC measures 2-4 % shorter, not equally for every tile
        from .measure import resnet_blob
        self.blob = pinned_like(resnet_blob(ctx, mid, 0, "fp16"))
        self.n_models = 1

    def _define(self, batch, table):
        from .runner import Worker
        if self.n_models > 400:   # models are never deleted from a context: start a new one now and then
            self.wk.close()
            self.wk = Worker(**POOLS)
            self.n_models = 0
        ctx = self.wk.ctx
        ctx.set_plan_table(rows(table))
        self.n_models += 1
        return ctx.model_define(self.ops, 3, self.hw, self.hw, batch_sizes=(batch,))

    def resnet_shapes(self, depth, batches=(1, 2, 4, 8, 16)):
        """Shape keys of every table-driven convolution launch of a ResNet at the given batch sizes."""
        ctx = self.wk.ctx
        ctx.set_plan_table([])
        mid = ctx.model_define_resnet(depth, self.hw, self.hw)
        ops = ctx.model_get_ops(mid)
        keys = set()
        for batch in batches:
            for l in ctx.plan(mid, batch):
                if l["kind"] == 1 and l["fused_op"] < 0:
                    o = ops[l["op_index"]]
                    keys.add((l["gemm_m"], l["gemm_n"], l["gemm_k"], o[3], o[5]))
        return keys

    def plan_choices(self, batch):
        """{shape key: (tile index, split)} as the library plans this batch size now."""
        mid = self._define(batch, {})
        out = {}
        for l in self.wk.ctx.plan(mid, batch):
            # a fused launch has its own fixed tile; a pair launch runs on the tile of its second member's
            # shape (the one reported here), so that row is tuned like any other
            if l["kind"] != 1 or l["fused_op"] >= 0:
                continue
            o = self.ops[l["op_index"]]
            key = (l["gemm_m"], l["gemm_n"], l["gemm_k"], o[3], o[5])   # M, N, K, kh, stride
            out[key] = (l["conv_tile"], l["split_k"])
        return out

    def measure(self, batch, table):
        """Median on-device EXEC duration (us) with `table` installed."""
        mid = self._define(batch, table)
        ctx = self.wk.ctx
        ctx.load_weights(mid, self.blob, self.wk.stream)
        self.wk.stream.synchronize()
        ctx.profile_measure(mid, batch, 8)
        p = ctx.profile_measure(mid, batch, self.reps)
        ctx.unload_weights(mid)
        return p["p50_us"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--family", default="resnet", choices=["resnet", "mobilenet", "densenet", "inception"],
                    help="resnet (of --depth) or one of measure.py's operator lists of the other families")
    ap.add_argument("--depth", type=int, default=50)
    ap.add_argument("--hw", type=int, default=224)
    ap.add_argument("--batches", default="1,2,4,8,16")
    ap.add_argument("--reps", type=int, default=60)
    ap.add_argument("--eps", type=float, default=0.2, help="a candidate must win by this many us")
    ap.add_argument("--kh", type=int, default=0, help="only retune shapes with this filter size (the others keep the library's choice)")
    ap.add_argument("--only-suffix", default="", help="only try tiles whose name ends like this")
    ap.add_argument("--verbose", action="store_true", help="print every candidate's time")
    ap.add_argument("--out", default=TABLE)
    ap.add_argument("--keep-existing", action="store_true", help="rows already in the output file are not replaced")
    ap.add_argument("--protect-resnet", type=int, default=0, help="shapes that this ResNet depth uses are neither retuned nor replaced")
    args = ap.parse_args()
    from .binding import CONV_TILES
    b = Bench(args.family, args.depth, args.hw, args.reps)
    protected = b.resnet_shapes(args.protect_resnet) if args.protect_resnet else set()
    final = {}
    for batch in (int(v) for v in args.batches.split(",")):
        t_start = time.time()
        cur = b.plan_choices(batch)
        t0 = b.measure(batch, cur)
        print("batch %d: %d shapes, start %.1f us" % (batch, len(cur), t0), flush=True)
        for key in sorted(cur, key=lambda k: -k[0] * k[1] * k[2]):
            best, best_t = cur[key], b.measure(batch, cur)
            if (args.kh and key[3] != args.kh) or key in protected:
                continue
            for tile, s in candidates(*key):
                if args.only_suffix and not tile.endswith(args.only_suffix):
                    continue
                cand = (CONV_TILES[tile], s)
                if cand == cur[key]:
                    continue
                t = b.measure(batch, {**cur, key: cand})
                if args.verbose:
                    print("      %s %s split %d: %.1f us (incumbent %.1f)" % (key, tile, s, t, best_t), flush=True)
                if t < best_t - args.eps:
                    best, best_t = cand, t
            if best != cur[key]:
                # confirm against a fresh measurement of the incumbent before switching
                if b.measure(batch, {**cur, key: best}) < b.measure(batch, cur) - args.eps / 2:
                    cur[key] = best
            print("  %s -> tile %d split %d   (EXEC %.1f us)" % (key, cur[key][0], cur[key][1], best_t), flush=True)
        t1 = b.measure(batch, cur)
        print("batch %d: %.1f -> %.1f us in %.0f s" % (batch, t0, t1, time.time() - t_start), flush=True)
        final.update(cur)
    b.wk.close()
    names = {v: k for k, v in CONV_TILES.items()}
    # rows of the table being rewritten whose shapes this run did not visit stay; with --keep-existing
    # the rows it did visit stay as well and only new shapes are added (a second model's own shapes
    # without moving the first model's choices)
    kept = read_table(args.out) if os.path.exists(args.out) else {}
    for key, val in kept.items():
        if key not in final or args.keep_existing or key in protected:
            final[key] = val
    lines = ["// Generated by paper_2006_02464_amd/tune.py on an MI355X: per GEMM shape the (tile, split-K) under which",
             "// whole EXECs ran fastest.  ResNet-50's shapes first; the shapes that only ResNet-18 or the MobileNet-,",
             "// DenseNet- and Inception-style lists have were added afterwards without moving those.",
             "// {M, N, K, kh, stride, tile, split_k}"]
    for key in sorted(final):
        tile, split = final[key]
        lines.append("{%d, %d, %d, %d, %d, %d, %d},  // %s" % (key + (tile, split, names[tile])))
    with open(args.out, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote %s (%d shapes)" % (args.out, len(final)))


if __name__ == "__main__":
    sys.exit(main())
