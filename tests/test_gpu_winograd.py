"""The Winograd F(2x2, 3x3) path (cw_set_winograd) against the CPU oracle, whose convolution is the
plain definition.  Winograd rounds three more tensors to the storage type (transformed input,
transformed weights, the 16 products) and cancels large terms in its output transform, so a layer
may differ from the direct kernel by a few storage ulps of the layer's largest value: the
teacher-forced bound here is 2 such ulps (measured: 0.87 in fp16, 0.99 in bf16), and the logits must still meet the
same per-sample tolerance as the direct path."""
import os

import numpy as np
import pytest

from gpu_common import TOL, Case, rel_err_per_sample
from oracle import network as N
from oracle import topology as T
from test_gpu_parity_full import GOLDEN, _per_sample
from workload import gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def worker():
    from paper_2006_02464_amd.runner import Worker
    w = Worker(workspace_bytes=2 << 30, io_bytes=256 << 20, weight_pool_bytes=1 << 30, load_staging_bytes=256 << 20)
    yield w
    w.close()


def _define(worker, ops, hw, batches, dtype="fp16", keep=False):
    ctx = worker.ctx
    ctx.set_winograd(1)
    ctx.set_debug_keep(keep)
    try:
        return ctx.model_define(ops, 3, hw, hw, batch_sizes=batches, dtype=dtype)
    finally:
        ctx.set_winograd(0)
        ctx.set_debug_keep(False)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_winograd_layers_against_the_oracle(worker, dtype):
    """ResNet-18 at 64x64 (odd tile counts in the last stages: 2x2 and 4x4 maps), batch 3: every
    3x3 stride-1 convolution runs as Winograd; each is compared with the oracle's convolution of the
    inputs the GPU produced."""
    case = Case(T.resnet(18), 72, seed=6, dtype=dtype, dist="uniform")      # 72 -> 18, 9, 5, 3: odd maps, ragged tiles
    mid = _define(worker, case.ops, 72, (3,), dtype, keep=True)
    plan = worker.ctx.plan(mid, 3)
    wino_ops = sorted({l["op_index"] for l in plan if l["name"] == "winograd_16gemms"})
    assert len(wino_ops) == 13 and all(case.ops[i].kh == 3 and case.ops[i].stride == 1 for i in wino_ops)
    assert sum(l["name"] == "winograd_16gemms" and l["grid_z"] == 16 for l in plan) == 13
    worker.load(mid, case.blob)
    x = case.images(0, 3)
    probs, logits, _ = worker.infer(mid, x)
    shapes = T.shapes(case.ops, 72, 72)
    ulp = 2.0 ** -10 if dtype == "fp16" else 2.0 ** -7
    gpu, wi, worst = {}, 0, 0.0
    for i, (o, (c, h, w)) in enumerate(zip(case.ops, shapes)):
        if o.op in (T.FC, T.SOFTMAX, T.GAVGPOOL):
            break
        gpu[i] = worker.ctx.debug_read_op(mid, 3, i, (3, c, h, w))
        if o.op == T.CONV:
            if i in wino_ops:
                src = gpu[o.input_from]
                t = _per_sample(lambda s: N.conv2d(s, case.w[wi], case.b[wi], o.stride, o.pad), src)
                if o.residual_from >= 0:
                    t = N.add(t, gpu[o.residual_from])
                if o.relu:
                    t = N.relu(t)
                t = gen.quantize(t, dtype)
                scale = np.abs(t).max()
                d = np.abs(gpu[i] - t).max() / (ulp * scale)
                worst = max(worst, float(d))
                assert d <= 2.0, "op %d: Winograd differs by %.2f storage ulps of the layer's largest value" % (i, d)
            wi += 1
    ref = case.oracle(x)["logits"]
    err = rel_err_per_sample(logits, ref)
    print("winograd resnet18 %s: 13 layers, worst teacher-forced diff %.2f ulps of the layer maximum; logits max rel err %.3e" % (dtype, worst, err.max()))
    assert err.max() <= TOL
    assert np.abs(probs - N.softmax(logits)).max() <= 1e-6
    worker.ctx.unload_weights(mid)


def test_winograd_resnet50_batch16_logits_and_time(worker):
    """ResNet-50 at 224x224, batch 16: the 13 stride-1 3x3 convolutions as Winograd; logits against
    the stored oracle logits; EXEC time next to the direct plan's."""
    case = Case(T.resnet(50), 224, seed=0, dist="normal")
    ref = np.load(os.path.join(GOLDEN, "resnet50_fp16_seed0_images0-1023_logits.npy"))[:16]
    wino = _define(worker, case.ops, 224, (16,))
    direct = worker.ctx.model_define(case.ops, 3, 224, 224, batch_sizes=(16,))
    assert sum(l["name"] == "winograd_16gemms" for l in worker.ctx.plan(wino, 16)) == 13
    x = case.images(0, 16)
    times = {}
    for name, mid in (("winograd", wino), ("direct", direct)):
        worker.load(mid, case.blob)
        logits = worker.infer(mid, x)[1]
        err = rel_err_per_sample(logits, ref)
        times[name] = worker.ctx.profile_measure(mid, 16, 200)["p50_us"]
        print("resnet50 b16 %s: max rel err %.3e, EXEC p50 %.1f us, %d launches" % (name, err.max(), times[name], len(worker.ctx.plan(mid, 16))))
        assert np.isfinite(logits).all() and err.max() <= TOL
        assert np.array_equal(N.argmax(logits), N.argmax(ref))
        worker.ctx.unload_weights(mid)
