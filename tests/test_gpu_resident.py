"""Resident launches (cw_set_resident): a run of convolution layers as one launch of 256 workgroups,
the batch cut into 8 partitions that each stay on one XCD.  Same arithmetic per tile as the per-layer
kernels; checked against the CPU oracle layer by layer and on the logits, for repeatability, and
for the error word staying clear."""
import os

import numpy as np
import pytest

from gpu_common import TOL, Case, rel_err_per_sample
from oracle import network as N
from oracle import topology as T
from test_gpu_parity_full import GOLDEN, _head, check_every_launch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def worker():
    from paper_2006_02464_amd.runner import Worker
    w = Worker(workspace_bytes=2 << 30, io_bytes=256 << 20, weight_pool_bytes=1 << 30, load_staging_bytes=256 << 20)
    yield w
    w.close()


def _define(worker, ops, hw, batches, dtype="fp16", keep=False, mode=1):
    ctx = worker.ctx
    ctx.set_resident(mode)
    ctx.set_debug_keep(keep)
    try:
        return ctx.model_define(ops, 3, hw, hw, batch_sizes=batches, dtype=dtype)
    finally:
        ctx.set_resident(0)
        ctx.set_debug_keep(False)


def test_resident_resnet18_small_maps_every_layer(worker):
    """ResNet-18 at 64x64, batch 8 and 16: partitions of 1 and 2 images whose last stages are 2x2 maps
    (4 and 8 pixels per partition: ragged tiles everywhere), every layer teacher forced."""
    case = Case(T.resnet(18), 64, seed=0, dist="uniform")
    mid = _define(worker, case.ops, 64, (8, 16), keep=True)
    for batch in (8, 16):
        plan = worker.ctx.plan(mid, batch)
        assert [l["name"] for l in plan if l["name"].startswith("resident")] == ["resident_19convs"]
        assert len(plan) == 7
    worker.load(mid, case.blob)
    for batch in (16, 8):
        x = case.images(0, batch)
        probs, logits, ns = worker.infer(mid, x)          # exec_duration_ns raises if the launch gave up
        wp, wf, nf, gpu = check_every_launch(worker, case, mid, batch, x)
        feat = [v for i, v in gpu.items() if case.ops[i].op == T.GAVGPOOL][0]
        _head(case, feat, logits, probs)
        err = rel_err_per_sample(logits, case.oracle(x)["logits"])
        print("resident resnet18 b%d: exec %.1f us, max rel err %.3e, worst teacher-forced diff / scale %.2e" % (batch, ns / 1e3, err.max(), wp))
        assert err.max() <= TOL
    worker.ctx.unload_weights(mid)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_resident_resnet50_every_layer_and_logits(worker, dtype):
    case = Case(T.resnet(50), 224, seed=0, dtype=dtype, dist="normal")
    mid = _define(worker, case.ops, 224, (16, 8), dtype, keep=True)
    assert [l["name"] for l in worker.ctx.plan(mid, 16) if l["kind"] == 11] == ["resident_52convs"]
    worker.load(mid, case.blob)
    x = case.images(0, 16)
    ref = np.load(os.path.join(GOLDEN, "resnet50_fp16_seed0_images0-1023_logits.npy"))[:16] if dtype == "fp16" else case.oracle(x)["logits"]
    for batch in (16, 8):
        got = []
        for i in range(0, 16, batch):
            probs, logits, ns = worker.infer(mid, x[i:i + batch])
            got.append(logits)
        wp, wf, nf, gpu = check_every_launch(worker, case, mid, batch, x[16 - batch:])
        feat = [v for i, v in gpu.items() if case.ops[i].op == T.GAVGPOOL][0]
        _head(case, feat, logits, probs)
        got = np.concatenate(got)
        err = rel_err_per_sample(got, ref)
        print("resident resnet50 %s b%d: exec %.1f us, max rel err %.3e, worst teacher-forced diff / scale %.2e" % (dtype, batch, ns / 1e3, err.max(), wp))
        assert np.isfinite(got).all() and err.max() <= TOL
        assert np.array_equal(N.argmax(got), N.argmax(ref))
    worker.ctx.unload_weights(mid)


def test_resident_later_stages_beside_fused_and_pair_launches(worker):
    """Mode 2: stages 3 and 4 of ResNet-50 as two resident launches, stages 1 and 2 as the fused
    and pair launches of the default plan; every layer teacher forced, logits against the oracle."""
    case = Case(T.resnet(50), 224, seed=0, dist="normal")
    mid = _define(worker, case.ops, 224, (16, 8), keep=True, mode=2)
    plan = worker.ctx.plan(mid, 16)
    assert [l["name"] for l in plan if l["kind"] == 11] == ["resident_17convs", "resident_8convs"]
    assert sum(l["fused_op"] >= 0 and l["kind"] == 1 for l in plan) == 7 and sum(l["pair_op"] >= 0 for l in plan) == 3
    worker.load(mid, case.blob)
    x = case.images(0, 16)
    ref = np.load(os.path.join(GOLDEN, "resnet50_fp16_seed0_images0-1023_logits.npy"))[:16]
    for batch in (16, 8):
        got = np.concatenate([worker.infer(mid, x[i:i + batch])[1] for i in range(0, 16, batch)])
        wp, wf, nf, gpu = check_every_launch(worker, case, mid, batch, x[16 - batch:])
        err = rel_err_per_sample(got, ref)
        print("resident (later stages) resnet50 b%d: %d launches, max rel err %.3e" % (batch, len(worker.ctx.plan(mid, batch)), err.max()))
        assert err.max() <= TOL
    worker.ctx.unload_weights(mid)


def test_resident_is_repeatable_and_timed_against_the_per_layer_plan(worker):
    """30 EXECs over one input give bit-identical logits (static tile assignment, fixed summation
    order); the EXEC time is printed next to the per-layer plan's."""
    case = Case(T.resnet(50), 224, seed=0, dist="normal")
    res = _define(worker, case.ops, 224, (16, 8))
    per_layer = worker.ctx.model_define(case.ops, 3, 224, 224, batch_sizes=(16, 8))
    x = case.images(0, 16)
    for name, mid in (("resident", res), ("per-layer", per_layer)):
        worker.load(mid, case.blob)
        first = worker.infer(mid, x)[1]
        if name == "resident":
            for _ in range(30):
                assert np.array_equal(worker.infer(mid, x)[1], first)
        for batch in (16, 8):
            p = worker.ctx.profile_measure(mid, batch, 300)
            print("resnet50 b%d %s: EXEC p50 %.1f us, p99 %.1f, max %.1f; %d launches" % (
                batch, name, p["p50_us"], p["p99_us"], p["max_us"], len(worker.ctx.plan(mid, batch))))
        worker.ctx.unload_weights(mid)
