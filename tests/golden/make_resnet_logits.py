"""Writes the stored oracle logits the GPU parity tests compare against.

Calls only the CPU oracle (``oracle/``) and the seeded input generator
(``workload/gen.py``); nothing here touches the HIP library.  Run from the
repository root:

    python tests/golden/make_resnet_logits.py [--threads N]

Outputs (float32 ``.npy``, loaded with ``numpy.load``):

* ``resnet50_fp16_seed0_images0-1023_logits.npy``  [1024][1000]
  ResNet-50 at 224x224, weights seed 0 rounded to fp16, images 0..1023 of image
  set seed 0, ~N(0,1), rounded to fp16: the 1024-sample parity set of the
  batch-1..16 workload (per-sample tolerance and top-1 agreement need at least
  a thousand samples to resolve 0.1 %).
* ``resnet152_bf16_seed0_images0-15_logits.npy``  [16][1000]
  ResNet-152 at 224x224, bf16 weights and images (fp16 overflows in this net
  without normalisation), one batch of 16.

Both are the plain definition in fp32 (oracle/oracle.c, nested loops); one
image per host thread, loops untouched.  Work is saved every chunk, so an
interrupted run resumes.  ResNet-50: ~8.2 GFLOP of scalar loops per image,
about 25 minutes for the 1024 images on 8 cores.
"""
import argparse
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)

from oracle import network as N   # noqa: E402
from oracle import topology as T  # noqa: E402
from workload import gen           # noqa: E402

SETS = {
    "resnet50": dict(depth=50, dtype="fp16", seed=0, count=1024,
                     path=os.path.join(HERE, "resnet50_fp16_seed0_images0-1023_logits.npy")),
    "resnet152": dict(depth=152, dtype="bf16", seed=0, count=16,
                      path=os.path.join(HERE, "resnet152_bf16_seed0_images0-15_logits.npy")),
}


def make(name, threads, chunk):
    s = SETS[name]
    ops = T.resnet(s["depth"])
    w, b = gen.model_tensors(T.weight_shapes(ops), s["seed"], s["dtype"])
    part = s["path"] + ".partial.npz"
    out = np.zeros((s["count"], 1000), np.float32)
    done = 0
    if os.path.exists(part):
        z = np.load(part)
        done = int(z["done"])
        out[:done] = z["logits"][:done]
    t0 = time.time()
    while done < s["count"]:
        n = min(chunk, s["count"] - done)
        x = gen.images(s["seed"], done, n, 3, 224, 224, "normal", s["dtype"])
        out[done:done + n] = N.forward(ops, w, b, x, prec="f32", threads=threads)["logits"]
        done += n
        np.savez(part, done=done, logits=out)
        print("%s: %d / %d images, %.0f s" % (name, done, s["count"], time.time() - t0), flush=True)
    np.save(s["path"], out)
    if os.path.exists(part):
        os.remove(part)


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--threads", type=int, default=len(os.sched_getaffinity(0)))
    ap.add_argument("--only", choices=sorted(SETS), default=None)
    a = ap.parse_args()
    for name in ([a.only] if a.only else ["resnet152", "resnet50"]):
        make(name, a.threads, chunk=4 * a.threads)
