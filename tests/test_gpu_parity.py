"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Tolerance: per sample, max_j |z_gpu - z_ref| <= 2e-2 *
max_j |z_ref| on the fp32 logits; top-1 is the lowest index attaining the maximum
on both sides."""
import numpy as np
import pytest

from gpu_common import TOL, Case, rel_err_per_sample, top2_gap
from workload import gen
from oracle import network as N
from oracle import topology as T

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def worker():
    from paper_2006_02464_amd.runner import Worker
    w = Worker(workspace_bytes=512 << 20, io_bytes=256 << 20, weight_pool_bytes=1 << 30,
               load_staging_bytes=256 << 20)
    yield w
    w.close()


def _layer_tol(dtype):
    # one rounding per stored activation: 2^-11 (fp16) / 2^-8 (bf16) relative to the layer's
    # magnitude, times a few layers of accumulated drift
    return 6e-3 if dtype == "fp16" else 4e-2


def check_all_ops(worker, case, mid, batch, x, teacher=True):
    """Every op's output against the oracle, two ways:

    * free running: the oracle's own same-index tensor, within a per-layer tolerance;
    * teacher forced: the oracle applies op i to the inputs the GPU actually produced for it
      (read back), then rounds once to the storage type.  The two can then differ only by
      summation order, i.e. by at most one unit in the last place of the storage type on the
      few elements that sit on a rounding boundary."""
    outs = case.oracle(x, keep="all")
    shapes = T.shapes(case.ops, case.hw, case.hw)
    ulp = 2.0 ** -10 if case.dtype == "fp16" else 2.0 ** -7
    worst = 0.0
    gpu = []
    wi = 0
    plan = worker.ctx.plan(mid, batch)
    # the first layer of a fused launch, and a projection computed inside one, are never stored
    unstored = ({l["fused_op"] for l in plan if l["kind"] in (1, 7) and l["fused_op"] >= 0} |
                {l["proj_op"] for l in plan if l["kind"] == 1 and l["proj_op"] >= 0})
    for i, (o, (c, h, w)) in enumerate(zip(case.ops, shapes)):
        if o.op in (T.FC, T.SOFTMAX):
            break
        if i in unstored:
            assert not teacher, "teacher forcing needs every tensor"
            gpu.append(None)
            wi += o.op == T.CONV
            continue
        shape = (batch, c) if o.op == T.GAVGPOOL else (batch, c, h, w)
        got = worker.ctx.debug_read_op(mid, batch, i, shape)
        gpu.append(got)
        ref = outs[i].reshape(shape)
        scale = np.abs(ref).max()
        err = np.abs(got - ref).max() / scale
        worst = max(worst, err)
        assert err <= _layer_tol(case.dtype), "op %d (%s): rel err %.3e" % (i, o, err)
        if not teacher:
            if o.op == T.CONV:
                wi += 1
            continue
        src = x if o.input_from < 0 else gpu[o.input_from]
        if o.op == T.CONV:
            t = N.conv2d(src, case.w[wi], case.b[wi], o.stride, o.pad)
            wi += 1
            if o.residual_from >= 0:
                t = N.add(t, gpu[o.residual_from])
            if o.relu:
                t = N.relu(t)
            t = gen.quantize(t, case.dtype)
            diff = np.abs(got - t)
            # an element on a rounding boundary may land one storage ulp away; sums that cancel
            # get an absolute allowance from the fp32 accumulation error of the layer
            allow = ulp * np.abs(t) + 1e-5 * scale
            assert (diff <= allow).all(), "op %d (%s): teacher-forced max diff %.3e" % (i, o, diff.max())
            assert (diff > 1e-5 * scale).mean() <= 0.02, "op %d: too many elements off by an ulp" % i
        elif o.op == T.MAXPOOL:
            assert np.array_equal(got, N.maxpool2d(src, o.kh, o.stride, o.pad)), "op %d: max pool not exact" % i
        elif o.op == T.GAVGPOOL:
            t = N.global_avgpool(src)
            assert np.abs(got - t).max() <= 1e-6 * np.abs(t).max()
    return outs, worst, gpu


def check_head(case, gpu_feat, logits, probs):
    """FC and softmax, teacher forced from the GPU's pooled features."""
    z = N.fc(gpu_feat, case.w[-1].reshape(case.w[-1].shape[0], -1), case.b[-1])
    assert np.abs(logits - z).max() <= 1e-5 * np.abs(z).max()
    assert np.abs(probs - N.softmax(logits)).max() <= 1e-6


# ---------------------------------------------------------------- config 1
def test_resnet18_64_batch1_every_layer(worker):
    """ResNet-18 at 64x64, batch 1, U[-1,1] input, seed 0: every layer and the logits."""
    case = Case(T.resnet(18), 64, seed=0, dist="uniform")
    worker.ctx.set_debug_keep(True)
    mid = worker.ctx.model_define_resnet(18, 64, 64)
    worker.ctx.set_debug_keep(False)
    worker.load(mid, case.blob)
    x = case.images(0, 1)
    probs, logits, ns = worker.infer(mid, x)
    outs, worst, gpu = check_all_ops(worker, case, mid, 1, x)
    check_head(case, gpu[-1], logits, probs)
    z_ref = outs[-2]
    assert rel_err_per_sample(logits, z_ref).max() <= TOL
    assert np.array_equal(N.argmax(logits), N.argmax(z_ref))
    assert ns > 0
    worker.ctx.unload_weights(mid)


@pytest.mark.parametrize("batch", [1, 2, 4, 8, 16])
def test_resnet18_all_batch_sizes_and_batch_invariance(worker, batch):
    case = Case(T.resnet(18), 64, seed=0, dist="uniform")
    mid = worker.ctx.model_define_resnet(18, 64, 64)
    worker.load(mid, case.blob)
    x = case.images(0, 16)
    ref = case.oracle(x)["logits"]
    got = np.concatenate([worker.infer(mid, x[i:i + batch])[1] for i in range(0, 16, batch)])
    assert rel_err_per_sample(got, ref).max() <= TOL
    assert np.array_equal(N.argmax(got), N.argmax(ref))
    worker.ctx.unload_weights(mid)


def test_resnet18_top1_agreement_2048_samples(worker):
    """Every sample within tolerance; top-1 agreement counted on 2048 samples.

    A random-weight network has near-ties: samples whose two largest oracle logits are closer
    than the fp16 storage error of the path.  Those may flip, and no summation order can avoid
    it (rounding stored activations to fp16 in the oracle itself moves its logits by as much).
    So: every mismatch must be such a near-tie (oracle top-2 gap <= 2x that sample's own
    logit error), agreement must be >= 99.9 % on the samples whose gap exceeds twice the
    largest logit error seen, and the raw rate is printed and bounded."""
    case = Case(T.resnet(18), 64, seed=0, dist="uniform")
    mid = worker.ctx.model_define_resnet(18, 64, 64)
    worker.load(mid, case.blob)
    n = 2048
    x = case.images(100, n)
    ref = case.oracle(x)["logits"]
    got = np.concatenate([worker.infer(mid, x[i:i + 16])[1] for i in range(0, n, 16)])
    err = rel_err_per_sample(got, ref)
    assert err.max() <= TOL
    a, b = N.argmax(got), N.argmax(ref)
    mism = np.nonzero(a != b)[0]
    abs_err = np.abs(got - ref).max(axis=1)
    gaps = top2_gap(ref)
    clear = gaps > 2 * abs_err.max()
    print("top-1 agreement %.4f (%d mismatches / %d); max rel err %.2e; well-separated samples %d, "
          "mismatches among them %d; (gap, err) of mismatches %s" % (
              1 - len(mism) / n, len(mism), n, err.max(), int(clear.sum()), int((a != b)[clear].sum()),
              [(float(gaps[i]), float(abs_err[i])) for i in mism]))
    from test_gpu_parity_full import _report
    _report("resnet18_64_2048", {"samples": n, "top1_agreement": 1 - len(mism) / n, "mismatches": [
        {"sample": int(i), "oracle_top2_gap": float(gaps[i]), "abs_err": float(abs_err[i])} for i in mism],
        "max_rel_err": float(err.max()), "well_separated_samples": int(clear.sum()),
        "mismatches_among_well_separated": int((a != b)[clear].sum()), "oracle_linf_median": float(np.median(np.abs(ref).max(axis=1))),
        "distinct_top1_classes": int(len(set(b.tolist())))})
    assert all(gaps[i] <= 2 * abs_err[i] for i in mism)      # only near-ties may flip
    assert (a != b)[clear].sum() <= clear.sum() // 1000
    assert len(mism) <= 0.005 * n
    # the oracle's own 16-bit-storage mode is as far from its fp32 mode as the GPU is
    ref16 = case.oracle(x[:256], storage="fp16")["logits"]
    print("fp16-storage oracle vs fp32 oracle: max rel err %.2e; GPU vs fp16-storage oracle %.2e" % (
        rel_err_per_sample(ref16, ref[:256]).max(), rel_err_per_sample(got[:256], ref16).max()))
    worker.ctx.unload_weights(mid)


# ---------------------------------------------------------------- every conv instantiation
@pytest.mark.parametrize("tile", ["128x128", "128x64", "64x64", "64x32", "32x64", "32x32",
                                  "128x64w2", "64x128w2", "256x64", "128x128w8",
                                  "128x64k128", "64x64k128", "64x32k128", "32x64k128", "32x32k128",
                                  "128x64k128g2", "64x64k128g2", "64x64k128g4", "64x32k128g4", "32x64k128g4",
                                  "32x32k128g4", "32x32k128g8", "128x64g2", "64x64g2", "32x32g4",
                                  "256x128w8", "128x256w8", "256x256w8", "256x128"])
@pytest.mark.parametrize("split_k", [1, 3])
def test_every_conv_tile_and_split_k(worker, tile, split_k):
    """Forces one tile shape and split-K factor on every convolution of ResNet-18 at 64x64
    (M from 4*B to 1024*B rows: ragged tiles in both dimensions)."""
    case = Case(T.resnet(18), 64, seed=1, dist="uniform")
    worker.ctx.set_plan_override(tile, split_k)
    worker.ctx.set_debug_keep(True)
    worker.ctx.set_panels(split_k == 3)     # the split-K half of the cases also numbers its tiles in channel panels
    try:
        mid = worker.ctx.model_define(case.ops, 3, 64, 64, batch_sizes=(3,))
    finally:
        worker.ctx.set_plan_override(-1, 0)
        worker.ctx.set_debug_keep(False)
        worker.ctx.set_panels(0)
    worker.load(mid, case.blob)
    x = case.images(0, 3)
    probs, logits, _ = worker.infer(mid, x)
    outs, _, gpu = check_all_ops(worker, case, mid, 3, x)
    check_head(case, gpu[-1], logits, probs)
    assert rel_err_per_sample(logits, outs[-2]).max() <= TOL
    worker.ctx.unload_weights(mid)


# ---------------------------------------------------------------- shapes off the ResNet path
def test_small_custom_net_narrow_channels_and_odd_stride_stem(worker):
    """A net none of whose layers takes the main kernel: a 3x3 stride-1 first convolution (odd
    stride: the register-staged stem with 3 filter rows), Cin = 32 and Cin = 96 (K slices of 32),
    a 5x5 convolution, a residual over a 1x1.  Every layer teacher-forced against the oracle."""
    O = T.Op
    ops = [
        O(T.CONV, 3, 32, 3, 3, 1, 1, 1, -1, -1),        # 0  first conv, stride 1
        O(T.CONV, 32, 96, 3, 3, 1, 1, 1, -1, 0),        # 1  Cin 32
        O(T.CONV, 96, 64, 1, 1, 1, 0, 1, -1, 1),        # 2  Cin 96, 1x1
        O(T.MAXPOOL, 64, 64, 3, 3, 2, 1, 0, -1, 2),     # 3
        O(T.CONV, 64, 96, 5, 5, 2, 2, 1, -1, 3),        # 4  5x5 stride 2 (main kernel, 25 taps)
        O(T.CONV, 96, 96, 3, 3, 1, 1, 0, -1, 4),        # 5  Cin 96, no activation
        O(T.CONV, 96, 96, 1, 1, 1, 0, 1, 4, 5),         # 6  Cin 96 with a residual
        O(T.CONV, 96, 256, 3, 3, 2, 1, 1, -1, 6),       # 7
        O(T.GAVGPOOL, 256, 256, 0, 0, 1, 0, 0, -1, 7),  # 8
        O(T.FC, 256, 10, 1, 1, 1, 0, 0, -1, 8),         # 9
        O(T.SOFTMAX, 10, 10, 0, 0, 1, 0, 0, -1, 9),     # 10
    ]
    case = Case(ops, 45, seed=5, dist="uniform")         # odd size: ragged rows and floor division
    worker.ctx.set_debug_keep(True)
    try:
        mid = worker.ctx.model_define(case.ops, 3, 45, 45, batch_sizes=(1, 5))
    finally:
        worker.ctx.set_debug_keep(False)
    plan = worker.ctx.plan(mid, 5)
    assert {l["tile_k"] for l in plan if l["kind"] == 1} == {32, 64}
    worker.load(mid, case.blob)
    for batch in (5, 1):
        x = case.images(0, batch)
        probs, logits, _ = worker.infer(mid, x, classes=10)
        outs, _, gpu = check_all_ops(worker, case, mid, batch, x)
        check_head(case, gpu[-1], logits, probs)
        assert rel_err_per_sample(logits, outs[-2]).max() <= TOL
    worker.ctx.unload_weights(mid)


@pytest.mark.parametrize("cout,dtype", [(64, "fp16"), (128, "fp16"), (128, "bf16")])
def test_max_pool_with_the_1x1_behind_it_every_layer(worker, cout, dtype):
    """The launch that computes a 3x3 max pool over 64 channels and the 1x1 convolution 64 -> 64 or 128
    behind it: 157 workgroups whose last holds 16 of 64 pixels, the pooled tensor (exact) and the
    convolution's output (teacher forced) against the oracle; a second convolution reads the pooled tensor too."""
    O = T.Op
    ops = [
        O(T.CONV, 3, 64, 7, 7, 2, 3, 1, -1, -1),           # 0
        O(T.MAXPOOL, 64, 64, 3, 3, 2, 1, 0, -1, 0),         # 1
        O(T.CONV, 64, cout, 1, 1, 1, 0, 1, -1, 1),          # 2  computed by the max pool's launch
        O(T.CONV, 64, 64, 3, 3, 1, 1, 1, -1, 1),            # 3  the pooled tensor's other reader
        O(T.CONV, cout, 256, 1, 1, 2, 0, 1, -1, 2),         # 4
        O(T.CONV, 64, 256, 1, 1, 2, 0, 1, 4, 3),            # 5  joins the two
        O(T.GAVGPOOL, 256, 256, 0, 0, 1, 0, 0, -1, 5),      # 6
        O(T.FC, 256, 10, 1, 1, 1, 0, 0, -1, 6),             # 7
        O(T.SOFTMAX, 10, 10, 0, 0, 1, 0, 0, -1, 7),         # 8
    ]
    case = Case(ops, 100, seed=9, dtype=dtype, dist="uniform")
    worker.ctx.set_debug_keep(True)
    try:
        mid = worker.ctx.model_define(case.ops, 3, 100, 100, batch_sizes=(16, 2), dtype=dtype)
    finally:
        worker.ctx.set_debug_keep(False)
    pool = [l for l in worker.ctx.plan(mid, 16) if l["kind"] == 3]
    assert len(pool) == 1 and pool[0]["fused_op"] == 2 and pool[0]["grid_x"] == 157 and pool[0]["gemm_n"] == cout
    assert [l["fused_op"] for l in worker.ctx.plan(mid, 2) if l["kind"] == 3] == [-1]     # 20 workgroups: two launches
    worker.load(mid, case.blob)
    for batch in (16, 2):
        x = case.images(0, batch)
        probs, logits, _ = worker.infer(mid, x, classes=10)
        outs, _, gpu = check_all_ops(worker, case, mid, batch, x)
        check_head(case, gpu[-1], logits, probs)
        assert rel_err_per_sample(logits, outs[-2]).max() <= TOL
    worker.ctx.unload_weights(mid)


@pytest.mark.parametrize("classes", [1500, 5000])
def test_pool_and_softmax_shapes_off_the_resnet_path(worker, classes):
    """A 2x2 max pool (the general window kernel, not the unrolled 3x3 one), a 5x5 average-pool
    map, and heads of 1500 and 5000 classes (softmax with 16 values per thread in registers, and
    the looping kernel for rows beyond 4096).  Every layer teacher-forced against the oracle."""
    O = T.Op
    ops = [
        O(T.CONV, 3, 64, 3, 3, 1, 1, 1, -1, -1),             # 0
        O(T.MAXPOOL, 64, 64, 2, 2, 2, 0, 0, -1, 0),          # 1  2x2 stride 2, no padding
        O(T.CONV, 64, 256, 3, 3, 2, 1, 1, -1, 1),            # 2
        O(T.GAVGPOOL, 256, 256, 0, 0, 1, 0, 0, -1, 2),       # 3
        O(T.FC, 256, classes, 1, 1, 1, 0, 0, -1, 3),         # 4
        O(T.SOFTMAX, classes, classes, 0, 0, 1, 0, 0, -1, 4),  # 5
    ]
    gain = [1.0, 1.0, 0.05]                                   # small logits: softmax not one-hot
    case = Case(ops, 20, seed=11, dist="uniform", weight_gain=gain)
    worker.ctx.set_debug_keep(True)
    try:
        mid = worker.ctx.model_define(case.ops, 3, 20, 20, batch_sizes=(1, 3))
    finally:
        worker.ctx.set_debug_keep(False)
    worker.load(mid, case.blob)
    for batch in (3, 1):
        x = case.images(0, batch)
        probs, logits, _ = worker.infer(mid, x, classes=classes)
        outs, _, gpu = check_all_ops(worker, case, mid, batch, x)
        check_head(case, gpu[-1], logits, probs)
        assert rel_err_per_sample(logits, outs[-2]).max() <= TOL
        assert probs.max() < 0.999                           # not one-hot: the sum over the row matters
        assert np.abs(probs - N.softmax(logits)).max() <= 1e-6
        assert np.abs(probs.sum(axis=1) - 1).max() <= 1e-5
    worker.ctx.unload_weights(mid)


@pytest.mark.parametrize("feat,classes,dtype", [(256, 1000, "fp16"), (768, 10, "fp16"), (512, 1024, "bf16"), (1024, 37, "fp16")])
def test_fc_and_softmax_in_one_launch(worker, feat, classes, dtype):
    """FC + softmax as one launch (K split over 2 or 4 workgroups per 16 outputs, softmax by the
    workgroup that finishes last) against the oracle on moderate logits, against the two-launch
    plan, at batch 1, 5 and 16, and bit-identical over 100 EXECs (arrival order must not matter).
    256 and 768 features: two splits; 512 and 1024: four.  10 and 37 classes: ragged output tiles."""
    O = T.Op
    ops = [
        O(T.CONV, 3, 64, 3, 3, 2, 1, 1, -1, -1),
        O(T.CONV, 64, feat, 3, 3, 2, 1, 1, -1, 0),
        O(T.GAVGPOOL, feat, feat, 0, 0, 1, 0, 0, -1, 1),
        O(T.FC, feat, classes, 1, 1, 1, 0, 0, -1, 2),
        O(T.SOFTMAX, classes, classes, 0, 0, 1, 0, 0, -1, 3),
    ]
    case = Case(ops, 16, seed=13, dtype=dtype, dist="uniform", weight_gain=[1.0, 1.0, 0.05])
    ctx = worker.ctx
    ctx.set_debug_keep(True)
    try:
        two = ctx.model_define(case.ops, 3, 16, 16, batch_sizes=(1, 5, 16), dtype=dtype)
        ctx.set_fc_softmax(1)
        one = ctx.model_define(case.ops, 3, 16, 16, batch_sizes=(1, 5, 16), dtype=dtype)
    finally:
        ctx.set_debug_keep(False)
        ctx.set_fc_softmax(0)
    for batch in (16, 5, 1):
        p1, p2 = ctx.plan(one, batch), ctx.plan(two, batch)
        assert [l["name"] for l in p1][-1] == "fc+softmax" and p1[-1]["split_k"] == (4 if feat % 512 == 0 else 2)
        assert [l["name"] for l in p2][-2:] == ["fc", "softmax"] and len(p1) == len(p2) - 1
        x = case.images(0, batch)
        worker.load(two, case.blob)
        probs2, logits2, _ = worker.infer(two, x, classes=classes)
        ctx.unload_weights(two)
        worker.load(one, case.blob)
        probs, logits, _ = worker.infer(one, x, classes=classes)
        outs, _, gpu = check_all_ops(worker, case, one, batch, x)
        check_head(case, gpu[-1], logits, probs)
        assert probs.max() < 0.999 and np.abs(probs.sum(axis=1) - 1).max() <= 1e-5
        assert np.abs(logits - logits2).max() <= 1e-5 * np.abs(logits2).max()
        assert np.abs(probs - probs2).max() <= 1e-6
        for _ in range(100 if batch == 16 else 10):
            pr, lg, _ = worker.infer(one, x, classes=classes)
            assert np.array_equal(lg, logits) and np.array_equal(pr, probs)
        ctx.unload_weights(one)


# ---------------------------------------------------------------- bf16
def test_resnet18_bf16(worker):
    case = Case(T.resnet(18), 64, seed=2, dtype="bf16", dist="uniform")
    worker.ctx.set_debug_keep(True)
    mid = worker.ctx.model_define_resnet(18, 64, 64, dtype="bf16")
    worker.ctx.set_debug_keep(False)
    worker.load(mid, case.blob)
    x = case.images(0, 4)
    probs, logits, _ = worker.infer(mid, x)
    outs, _, gpu = check_all_ops(worker, case, mid, 4, x)
    check_head(case, gpu[-1], logits, probs)
    assert rel_err_per_sample(logits, outs[-2]).max() <= TOL
    worker.ctx.unload_weights(mid)


# ---------------------------------------------------------------- softmax on moderate logits
def test_softmax_against_oracle_on_small_logits(worker):
    """With real He-normal weights the logits are ~1e3 and softmax is one-hot, so the
    probabilities are compared on a model whose FC weights are scaled down."""
    ops = T.resnet(18)
    gain = [1.0] * len(T.weight_shapes(ops))
    gain[-1] = 0.02
    case = Case(ops, 64, seed=3, dist="uniform", weight_gain=gain)
    mid = worker.ctx.model_define_resnet(18, 64, 64)
    worker.load(mid, case.blob)
    x = case.images(0, 8)
    probs, logits, _ = worker.infer(mid, x)
    ref = case.oracle(x)
    assert np.abs(ref["logits"]).max() < 30
    assert ref["probs"].max() < 0.999               # not one-hot
    # softmax of the GPU's own logits, by the oracle: isolates the softmax kernel
    assert np.abs(probs - N.softmax(logits)).max() <= 1e-6
    assert np.abs(probs.sum(axis=1) - 1).max() <= 1e-5
    assert np.array_equal(N.argmax(probs), N.argmax(logits))
    # end to end: |dp| <= |dz|_inf * 2 * p  (softmax is 1-Lipschitz-ish); loose check
    dz = np.abs(logits - ref["logits"]).max()
    assert np.abs(probs - ref["probs"]).max() <= 2.5 * dz + 1e-6
    worker.ctx.unload_weights(mid)


# ---------------------------------------------------------------- config 2
@pytest.fixture(scope="module")
def r50():
    case = Case(T.resnet(50), 224, seed=0, dist="normal")
    x = case.images(0, 16)
    ref = case.oracle(x)["logits"]       # 16 images, one per host thread
    return case, x, ref


def test_resnet50_224_batch16(worker, r50):
    case, x, ref = r50
    mid = worker.ctx.model_define_resnet(50, 224, 224)
    worker.load(mid, case.blob)
    probs, logits, ns = worker.infer(mid, x)
    err = rel_err_per_sample(logits, ref)
    print("resnet50 b16: max rel err %.3e, |z|inf %.1f, exec %.1f us" % (err.max(), np.abs(ref).max(), ns / 1e3))
    assert np.isfinite(logits).all()
    assert err.max() <= TOL
    assert np.array_equal(N.argmax(logits), N.argmax(ref))
    assert np.abs(probs.sum(axis=1) - 1).max() <= 1e-5
    assert np.array_equal(N.argmax(probs), N.argmax(logits))
    # same input twice: bit-identical (fixed summation order, no atomics)
    _, again, _ = worker.infer(mid, x)
    assert np.array_equal(again, logits)
    worker.ctx.unload_weights(mid)


def test_resnet50_fused_and_unfused_plans_agree(worker, r50):
    """Batch 16 and 8 plan the 3x3 + 1x1 tail of the early bottlenecks as one launch.  Both plans
    must meet the tolerance against the oracle, and they compute the same sums in the same order
    (the intermediate is rounded to the storage type either way; only a projection shortcut folded
    into the launch skips its rounding), so they should agree far more closely than either does
    with the fp32 oracle."""
    case, x, ref = r50
    ctx = worker.ctx
    fused = ctx.model_define_resnet(50, 224, 224)      # default: two wave groups where the first layer has 128 channels
    try:
        ctx.set_fusion(2)
        fused1 = ctx.model_define_resnet(50, 224, 224)  # one wave group
        ctx.set_fusion(0)
        plain = ctx.model_define_resnet(50, 224, 224)
    finally:
        ctx.set_fusion(1)
    for batch in (16, 8):
        blocks = {name: sorted({l["block"] for l in ctx.plan(mid, batch) if l["fused_op"] >= 0 and l["kind"] == 1})
                  for name, mid in (("fused", fused), ("fused1", fused1), ("plain", plain))}
        # two groups of four waves for the 128-channel pairs (stage 2), one group for the 64-channel ones
        assert blocks == {"fused": [256, 512], "fused1": [256], "plain": []}
        n_fused = sum(l["fused_op"] >= 0 and l["kind"] == 1 for l in ctx.plan(fused, batch))
        out = {}
        for name, mid in (("fused", fused), ("fused1", fused1), ("plain", plain)):
            worker.load(mid, case.blob)
            out[name] = np.concatenate([worker.infer(mid, x[i:i + batch])[1] for i in range(0, 16, batch)])
            ctx.unload_weights(mid)
            assert rel_err_per_sample(out[name], ref).max() <= TOL
            assert np.array_equal(N.argmax(out[name]), N.argmax(ref))
        d = max(rel_err_per_sample(out[k], out["plain"]).max() for k in ("fused", "fused1"))
        print("batch %d: %d fused launches, fused vs plain max rel diff %.3e" % (batch, n_fused, d))
        # the same products, summed per wave group where there are two; a projection shortcut
        # computed inside a fused launch is not rounded to the storage type on its way into the sum
        assert d <= 5e-3


def test_resnet50_pair_launches_change_nothing(worker, r50):
    """The first 1x1 of a block and the projection shortcut beside it as one launch or as two: the same
    products; a member may run on the other's tile shape, whose K slices and wave groups add them up
    in another order, so the two plans agree to rounding, far closer than either to the fp32 oracle."""
    case, x, ref = r50
    ctx = worker.ctx
    paired = ctx.model_define_resnet(50, 224, 224)
    ctx.set_pair_launches(0)
    try:
        single = ctx.model_define_resnet(50, 224, 224)
    finally:
        ctx.set_pair_launches(1)
    for batch in (16, 1):
        n = 16 if batch == 16 else 4
        assert sum(l["pair_op"] >= 0 for l in ctx.plan(paired, batch)) >= 3
        assert not any(l["pair_op"] >= 0 for l in ctx.plan(single, batch))
        out = {}
        for name, mid in (("paired", paired), ("single", single)):
            worker.load(mid, case.blob)
            out[name] = np.concatenate([worker.infer(mid, x[i:i + batch])[1] for i in range(0, n, batch)])
            ctx.unload_weights(mid)
        assert rel_err_per_sample(out["paired"], ref[:n]).max() <= TOL
        d = rel_err_per_sample(out["paired"], out["single"]).max()
        print("batch %d: paired vs single launches max rel diff %.3e" % (batch, d))
        assert d <= 5e-3


def test_resnet50_max_pool_with_its_1x1_changes_nothing(worker, r50):
    """The max pool and the first bottleneck's 1x1 reduce as one launch or as two: the pooled values are
    exact either way and the 64-deep products are added in the same order, so the logits are the same bits."""
    case, x, ref = r50
    ctx = worker.ctx
    one = ctx.model_define_resnet(50, 224, 224)
    ctx.set_fusion_pool(0)
    try:
        two = ctx.model_define_resnet(50, 224, 224)
    finally:
        ctx.set_fusion_pool(1)
    for batch in (16, 2):
        n = 16 if batch == 16 else 4
        pool = [l for l in ctx.plan(one, batch) if l["kind"] == 3]
        assert len(pool) == 1 and pool[0]["fused_op"] == 2 and pool[0]["name"] == "maxpool3x3_s2+1x1"
        assert [l["fused_op"] for l in ctx.plan(two, batch) if l["kind"] == 3] == [-1]
        assert len(ctx.plan(two, batch)) == len(ctx.plan(one, batch)) + 1
        out = {}
        for name, mid in (("one", one), ("two", two)):
            worker.load(mid, case.blob)
            out[name] = np.concatenate([worker.infer(mid, x[i:i + batch])[1] for i in range(0, n, batch)])
            ctx.unload_weights(mid)
        assert rel_err_per_sample(out["one"], ref[:n]).max() <= TOL
        assert np.array_equal(out["one"], out["two"])
    assert not [l for l in ctx.plan(one, 1) if l["kind"] == 3 and l["fused_op"] >= 0]   # too few workgroups at batch 1


def test_resnet50_panel_numbering_changes_nothing(worker, r50):
    """Numbering a launch's tiles in channel panels only changes which workgroup computes which
    tile: the logits are bit-identical to the default plan's, at batch 16 (panels of 2, 4 and 8 in
    stages 3-4, pair launches included) and at batch 1 (split-K launches included)."""
    case, x, ref = r50
    ctx = worker.ctx
    rows = ctx.model_define_resnet(50, 224, 224)
    ctx.set_panels(1)
    try:
        panels = ctx.model_define_resnet(50, 224, 224)
    finally:
        ctx.set_panels(0)
    for batch in (16, 1):
        n = 16 if batch == 16 else 4
        assert all(max(l["panels"] & 255, l["panels"] >> 8) <= 1 for l in ctx.plan(rows, batch))
        seen = {l["panels"] & 255 for l in ctx.plan(panels, batch)} | {l["panels"] >> 8 for l in ctx.plan(panels, batch)}
        assert {2, 4, 8} <= seen
        if batch == 1:
            assert any((l["panels"] & 255) > 1 and l["split_k"] > 1 for l in ctx.plan(panels, batch))
        out = {}
        for name, mid in (("rows", rows), ("panels", panels)):
            worker.load(mid, case.blob)
            out[name] = np.concatenate([worker.infer(mid, x[i:i + batch])[1] for i in range(0, n, batch)])
            ctx.unload_weights(mid)
        assert rel_err_per_sample(out["panels"], ref[:n]).max() <= TOL
        assert np.array_equal(out["panels"], out["rows"])


@pytest.mark.parametrize("batch", [1, 2, 4, 8])
def test_resnet50_224_small_batches(worker, r50, batch):
    case, x, ref = r50
    mid = worker.ctx.model_define_resnet(50, 224, 224)
    worker.load(mid, case.blob)
    n = min(16, 4 * batch)
    got = np.concatenate([worker.infer(mid, x[i:i + batch])[1] for i in range(0, n, batch)])
    assert rel_err_per_sample(got, ref[:n]).max() <= TOL
    assert np.array_equal(N.argmax(got), N.argmax(ref[:n]))
    worker.ctx.unload_weights(mid)


def test_resnet50_split_k_is_reproducible(worker, r50):
    """With K split over 4 workgroups in every layer, each tile is finished by whichever workgroup
    arrives last; the sum must not depend on that order: 200 EXECs, bit-identical logits.  The
    default batch-1 plan (wave groups inside a workgroup, a few split layers) likewise."""
    case, x, ref = r50
    worker.ctx.set_plan_override(-1, 4)
    try:
        split = worker.ctx.model_define_resnet(50, 224, 224)
    finally:
        worker.ctx.set_plan_override(-1, 0)
    default = worker.ctx.model_define_resnet(50, 224, 224)
    assert sum(l["split_k"] > 1 for l in worker.ctx.plan(split, 1)) >= 40
    base = {(128, 128): 256, (128, 64): 256, (64, 64): 256, (64, 32): 128, (32, 64): 128, (32, 32): 64, (256, 64): 256}
    grouped = [l for l in worker.ctx.plan(default, 1) if l["kind"] == 1 and
               (l["block"] > base[(l["tile_m"], l["tile_n"])] or l["split_k"] > 1)]
    assert len(grouped) >= 10   # several waves (or workgroups) add up one tile
    for mid, reps in ((split, 200), (default, 50)):
        worker.load(mid, case.blob)
        first = worker.infer(mid, x[:1])[1]
        assert rel_err_per_sample(first, ref[:1]).max() <= TOL
        for _ in range(reps):
            assert np.array_equal(worker.infer(mid, x[:1])[1], first)
        worker.ctx.unload_weights(mid)


def test_resnet50_first_block_every_layer(worker):
    """Per-layer parity on the real 224x224 shapes (stem, max pool, first bottleneck, and on
    through the network) at batch 2."""
    case = Case(T.resnet(50), 224, seed=5, dist="normal")
    worker.ctx.set_debug_keep(True)
    mid = worker.ctx.model_define(case.ops, 3, 224, 224, batch_sizes=(2,))
    worker.ctx.set_debug_keep(False)
    worker.load(mid, case.blob)
    x = case.images(0, 2)
    probs, logits, _ = worker.infer(mid, x)
    outs, worst, gpu = check_all_ops(worker, case, mid, 2, x, teacher=False)
    check_head(case, gpu[-1], logits, probs)
    print("worst per-layer rel err %.3e" % worst)
    assert rel_err_per_sample(logits, outs[-2]).max() <= TOL
    worker.ctx.unload_weights(mid)


# ---------------------------------------------------------------- config 4 (bf16: fp16 would overflow)
def test_resnet152_bf16_batch16_sampled(worker):
    """ResNet-152 at batch 16 in bf16 storage; the oracle checks 4 of the 16 samples (samples
    are independent, so each is computed on its own)."""
    case = Case(T.resnet(152), 224, seed=0, dtype="bf16", dist="normal")
    mid = worker.ctx.model_define_resnet(152, 224, 224, dtype="bf16")
    worker.load(mid, case.blob)
    x = case.images(0, 16)
    probs, logits, ns = worker.infer(mid, x)
    assert np.isfinite(logits).all()
    pick = [0, 5, 10, 15]
    ref = case.oracle(x[pick])["logits"]
    err = rel_err_per_sample(logits[pick], ref)
    print("resnet152 bf16 b16: max rel err %.3e, |z|inf %.3e, exec %.1f us" % (err.max(), np.abs(ref).max(), ns / 1e3))
    assert err.max() <= TOL
    worker.ctx.unload_weights(mid)
