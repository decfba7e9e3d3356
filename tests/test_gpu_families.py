"""GPU parity of the operators beyond the ResNet set (depthwise and rectangular convolution, hard
swish, CONCAT written in place) on the MobileNet-, DenseNet- and Inception-style operator lists:
every layer teacher forced against the CPU oracle, logits within the per-sample tolerance."""
import numpy as np
import pytest

from gpu_common import TOL, Case, rel_err_per_sample
from oracle import network as N
from oracle import topology as T
from test_gpu_parity_full import _head, check_every_launch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def worker():
    from paper_2006_02464_amd.runner import Worker
    w = Worker(workspace_bytes=2 << 30, io_bytes=256 << 20, weight_pool_bytes=512 << 20, load_staging_bytes=256 << 20)
    yield w
    w.close()


FAMILIES = {
    "mobilenet": (lambda: T.mobilenet(), 96),
    "dense": (lambda: T.dense_net(), 64),
    "inception": (lambda: T.inception_net(), 72),
}


@pytest.mark.parametrize("family", sorted(FAMILIES))
@pytest.mark.parametrize("dtype,batch", [("fp16", 3), ("bf16", 16), ("fp16", 16)])
def test_family_every_layer(worker, family, dtype, batch):
    make, hw = FAMILIES[family]
    case = Case(make(), hw, seed=21, dtype=dtype, dist="normal")
    ctx = worker.ctx
    ctx.set_debug_keep(True)
    try:
        mid = ctx.model_define(case.ops, 3, hw, hw, batch_sizes=(batch,), dtype=dtype)
    finally:
        ctx.set_debug_keep(False)
    plan = ctx.plan(mid, batch)
    kinds = {l["name"].split("_")[0].rstrip("0123456789x") for l in plan}
    if family == "mobilenet":
        assert sum(l["name"].startswith("dwconv") for l in plan) == 13
    if family == "dense":     # 18 CONCATs, only the two block inputs (max-pool outputs) are copied in
        assert sum(l["name"] == "concat_copy" for l in plan) == 2
    if family == "inception":  # both CONCATs are written in place; 1x7 and 7x1 run on the main kernel
        assert not any(l["name"] == "concat_copy" for l in plan)
        assert sum(l["name"].startswith(("conv1x7", "conv7x1")) for l in plan) == 4
    worker.load(mid, case.blob)
    x = case.images(0, batch)
    probs, logits, ns = worker.infer(mid, x)
    assert np.isfinite(logits).all()
    wp, wf, nf, gpu = check_every_launch(worker, case, mid, batch, x)
    feat = [v for i, v in gpu.items() if case.ops[i].op == T.GAVGPOOL][0]
    _head(case, feat, logits, probs)
    ref = case.oracle(x)["logits"]
    err = rel_err_per_sample(logits, ref)
    print("%s %s b%d: %d launches, exec %.1f us, max rel err %.3e, worst teacher-forced diff / scale %.2e" % (
        family, dtype, batch, len(plan), ns / 1e3, err.max(), wp), kinds)
    assert err.max() <= TOL
    ctx.unload_weights(mid)


def test_mobilenet_224_batch16_and_small_batches(worker):
    """The depthwise family at its real size: 224x224, batch 16 and re-cut at batch 1 and 4."""
    case = Case(T.mobilenet(), 224, seed=0, dist="normal")
    ctx = worker.ctx
    mid = ctx.model_define(case.ops, 3, 224, 224)
    worker.load(mid, case.blob)
    x = case.images(0, 16)
    ref = case.oracle(x)["logits"]
    for batch in (16, 4, 1):
        got = np.concatenate([worker.infer(mid, x[i:i + batch])[1] for i in range(0, 16, batch)])
        err = rel_err_per_sample(got, ref)
        print("mobilenet 224 b%d: max rel err %.3e, top-1 equal on %d of 16" % (batch, err.max(), int((N.argmax(got) == N.argmax(ref)).sum())))
        assert err.max() <= TOL
    p = ctx.profile_measure(mid, 16, 200)
    print("mobilenet 224 b16 EXEC p50 %.1f us" % p["p50_us"])
    ctx.unload_weights(mid)


@pytest.mark.parametrize("name", ["resnet18", "dense", "inception"])
def test_models_with_tuned_shapes_at_224(worker, name):
    """ResNet-18 and the DenseNet- and Inception-style lists at 224x224, where their convolution shapes
    have rows of their own in the plan table: batch 16, re-cut at batch 4 and 1, logits against the oracle."""
    make = {"resnet18": lambda: T.resnet(18), "dense": T.dense_net, "inception": T.inception_net}[name]
    case = Case(make(), 224, seed=0, dist="normal")
    ctx = worker.ctx
    mid = ctx.model_define(case.ops, 3, 224, 224)
    worker.load(mid, case.blob)
    x = case.images(0, 16)
    ref = case.oracle(x)["logits"]
    for batch in (16, 4, 1):
        got = np.concatenate([worker.infer(mid, x[i:i + batch])[1] for i in range(0, 16, batch)])
        err = rel_err_per_sample(got, ref)
        print("%s 224 b%d: %d launches, max rel err %.3e, top-1 equal on %d of 16" % (
            name, batch, len(ctx.plan(mid, batch)), err.max(), int((N.argmax(got) == N.argmax(ref)).sum())))
        assert np.isfinite(got).all() and err.max() <= TOL
    ctx.unload_weights(mid)


def test_mobilenet_depthwise_with_its_1x1_or_apart(worker):
    """The depthwise 3x3 convolutions over 32 and 64 channels inside the launch of the 1x1 behind them, or as
    launches of their own: the depthwise values are the same bits either way; the 1x1 adds its products up in
    another order than the stand-alone kernel that takes K = 32, so the plans agree to rounding."""
    case = Case(T.mobilenet(), 224, seed=0, dist="normal")
    ctx = worker.ctx
    fused = ctx.model_define(case.ops, 3, 224, 224)
    ctx.set_fusion_dw(0)
    try:
        apart = ctx.model_define(case.ops, 3, 224, 224)
    finally:
        ctx.set_fusion_dw(1)
    x = case.images(0, 8)
    ref = case.oracle(x)["logits"]
    for batch, n_fused in ((4, 2), (1, 1)):
        pl = ctx.plan(fused, batch)
        both = [l for l in pl if l["kind"] == 7 and l["fused_op"] >= 0]
        assert len(both) == n_fused and all(l["fused_op"] == l["op_index"] - 1 and l["name"].endswith("+1x1") for l in both)
        assert len(ctx.plan(apart, batch)) == len(pl) + n_fused and not [l for l in ctx.plan(apart, batch) if l["fused_op"] >= 0]
        out = {}
        for name, mid in (("fused", fused), ("apart", apart)):
            worker.load(mid, case.blob)
            out[name] = np.concatenate([worker.infer(mid, x[i:i + batch])[1] for i in range(0, 8, batch)])
            ctx.unload_weights(mid)
        assert rel_err_per_sample(out["fused"], ref).max() <= TOL
        d = rel_err_per_sample(out["fused"], out["apart"]).max()
        print("mobilenet b%d: fused vs apart max rel diff %.3e" % (batch, d))
        assert d <= 2e-3


def test_depthwise_shapes_off_the_mobilenet_path(worker):
    """Depthwise filters MobileNet does not have (5x5 padding 2 with hard swish, 3x3 without padding,
    3x3 stride 3) and 3x3 ones on odd map widths (19, 10, 8, 3 columns), one with a residual: every
    layer against the oracle."""
    O = T.Op
    ops = [
        O(T.CONV, 3, 64, 3, 3, 1, 1, 1, -1, -1),                 # 0   19x19
        O(T.CONV, 64, 64, 5, 5, 1, 2, 2, -1, 0, 0, 64),           # 1   5x5 depthwise, hard swish
        O(T.CONV, 64, 64, 3, 3, 1, 1, 1, 0, 1, 0, 64),            # 2   19 columns, residual
        O(T.CONV, 64, 64, 3, 3, 2, 1, 0, -1, 2, 0, 64),           # 3   stride 2 -> 10x10
        O(T.CONV, 64, 64, 3, 3, 1, 0, 1, -1, 3, 0, 64),           # 4   no padding -> 8x8
        O(T.CONV, 64, 64, 3, 3, 1, 1, 1, -1, 4, 0, 64),           # 5
        O(T.CONV, 64, 64, 3, 3, 3, 1, 1, -1, 5, 0, 64),           # 6   stride 3 -> 3x3
        O(T.CONV, 64, 256, 1, 1, 1, 0, 1, -1, 6),                 # 7
        O(T.GAVGPOOL, 256, 256, 0, 0, 1, 0, 0, -1, 7),
        O(T.FC, 256, 100, 1, 1, 1, 0, 0, -1, 8),
        O(T.SOFTMAX, 100, 100, 0, 0, 1, 0, 0, -1, 9),
    ]
    for dtype, batch in (("fp16", 5), ("bf16", 2)):
        case = Case(ops, 19, seed=31, dtype=dtype, dist="normal")
        ctx = worker.ctx
        ctx.set_debug_keep(True)
        try:
            mid = ctx.model_define(case.ops, 3, 19, 19, batch_sizes=(batch,), dtype=dtype)
        finally:
            ctx.set_debug_keep(False)
        assert sum(l["name"].startswith("dwconv") for l in ctx.plan(mid, batch)) == 6
        worker.load(mid, case.blob)
        x = case.images(0, batch)
        probs, logits, ns = worker.infer(mid, x, classes=100)
        wp, wf, nf, gpu = check_every_launch(worker, case, mid, batch, x)
        ref = case.oracle(x)["logits"]
        assert rel_err_per_sample(logits, ref).max() <= TOL
        ctx.unload_weights(mid)
