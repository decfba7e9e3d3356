"""Pins for the oracle's topology lists and whole-network forward pass (no GPU)."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import network as N
from oracle import topology as T
from workload import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_resnet_sizes.txt")


def _table1():
    rows = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        rows[f[0]] = [float(v) for v in f[1:]]
    return rows


@pytest.mark.parametrize("depth,params,macs,hw", [
    (18, 11_684_712, 148_557_824, 64),
    (50, 25_530_472, 4_089_184_256, 224),
    (152, 60_117_096, 11_513_626_624, 224),
])
def test_topology_counts(depth, params, macs, hw):
    ops = T.resnet(depth)
    # textbook parameter counts (11,689,512 / 25,557,032 / 60,192,808) minus one
    # BatchNorm vector per conv, which folding removes
    nconv = sum(o.op == T.CONV for o in ops)
    bn_channels = sum(o.cout for o in ops if o.op == T.CONV)
    textbook = {18: 11_689_512, 50: 25_557_032, 152: 60_192_808}[depth]
    assert T.param_count(ops) == textbook - bn_channels == params
    assert T.mac_count(ops, hw, hw) == macs
    assert nconv == {18: 20, 50: 53, 152: 155}[depth]


@pytest.mark.parametrize("depth", [18, 50, 152])
def test_topology_matches_paper_table1_sizes(depth):
    """Table 1: fp32 weight blob sizes, 602 kB input, 4 kB output."""
    row = _table1()["resnet%d" % depth]
    in_kb, out_kb, w_mb = row[0], row[1], row[2]
    ops = T.resnet(depth)
    assert abs(T.param_count(ops) * 4 / 1e6 - w_mb) / w_mb < 3e-3
    assert round(3 * 224 * 224 * 4 / 1e3) == in_kb
    assert ops[-1].cout * 4 / 1e3 == out_kb


def test_feature_map_sizes_resnet50():
    ops = T.resnet(50)
    shp = T.shapes(ops, 224, 224)
    assert shp[0] == (64, 112, 112) and shp[1] == (64, 56, 56)
    spatial = sorted({s[1] for s in shp[2:-3]}, reverse=True)
    assert spatial == [56, 28, 14, 7]
    assert shp[-4] == (2048, 7, 7) and shp[-3] == (2048, 1, 1) and shp[-2] == (1000, 1, 1)
    # config-1 shape: ResNet-18 at 64x64 ends on a 2x2 map
    assert T.shapes(T.resnet(18), 64, 64)[-4] == (512, 2, 2)


def _torch_resnet_forward(depth, weights, biases, x):
    """Independent float64 forward written with torch.nn.functional in the usual
    block structure (not by walking the op list)."""
    kind, blocks = {18: ("basic", [2, 2, 2, 2]), 50: ("bottleneck", [3, 4, 6, 3])}[depth]
    it = iter(zip(weights, biases))

    def conv(t, stride, pad):
        w, b = next(it)
        return F.conv2d(t, torch.from_numpy(w).double(), torch.from_numpy(b).double(),
                        stride=stride, padding=pad)

    t = torch.from_numpy(x).double()
    t = F.relu(conv(t, 2, 3))
    t = F.max_pool2d(t, 3, 2, 1)
    cin = 64
    for stage, (w, nb) in enumerate(zip([64, 128, 256, 512], blocks)):
        for b in range(nb):
            s = 2 if (b == 0 and stage > 0) else 1
            cout = w if kind == "basic" else 4 * w
            inp = t
            if kind == "basic":
                u = F.relu(conv(inp, s, 1))
            else:
                u = F.relu(conv(inp, 1, 0))
                u = F.relu(conv(u, s, 1))
            sc = inp
            if s != 1 or cin != cout:
                sc = conv(inp, s, 0)
            u = conv(u, 1, 1 if kind == "basic" else 0)
            t = F.relu(u + sc)
            cin = cout
    f = t.mean(dim=(2, 3))
    w, b = next(it)
    z = f @ torch.from_numpy(w.reshape(w.shape[0], -1)).double().T + torch.from_numpy(b).double()
    return z.numpy(), torch.softmax(z, dim=1).numpy()


@pytest.mark.parametrize("depth,hw", [(18, 64), (50, 32)])
def test_forward_vs_independent_torch_f64(depth, hw):
    ops = T.resnet(depth)
    w, b = gen.model_tensors(T.weight_shapes(ops), seed=3)
    x = gen.images(3, 0, 2, 3, hw, hw, "uniform")
    zt, pt = _torch_resnet_forward(depth, w, b, x)
    r64 = N.forward(ops, w, b, x, prec="f64")
    linf = np.abs(zt).max()
    assert np.abs(r64["logits"] - zt).max() <= 1e-11 * linf
    assert np.abs(r64["probs"] - pt).max() <= 1e-9
    r32 = N.forward(ops, w, b, x, prec="f32")
    assert np.abs(r32["logits"] - zt).max() <= 1e-5 * linf
    assert np.array_equal(N.argmax(r32["logits"]), zt.argmax(1))


@pytest.fixture(scope="module")
def r18():
    ops = T.resnet(18)
    w, b = gen.model_tensors(T.weight_shapes(ops), seed=0)
    return ops, w, b


def test_positive_homogeneity_exact(r18):
    """With all biases zero every op is positively homogeneous of degree 1, so a
    power-of-two input scale must scale the fp32 logits bit for bit."""
    ops, w, b = r18
    zb = [np.zeros_like(v) for v in b]
    x = gen.images(0, 0, 1, 3, 64, 64, "uniform")
    base = N.forward(ops, w, zb, x)["logits"]
    assert np.abs(base).max() > 0
    for k in (-3, 1, 4):
        sc = N.forward(ops, w, zb, x * np.float32(2.0 ** k))["logits"]
        assert np.array_equal(sc, base * np.float32(2.0 ** k))
        assert np.array_equal(N.argmax(sc), N.argmax(base))


def test_zero_input_zero_bias_gives_zero_logits(r18):
    ops, w, b = r18
    zb = [np.zeros_like(v) for v in b]
    r = N.forward(ops, w, zb, np.zeros((1, 3, 64, 64), np.float32))
    assert not r["logits"].any()
    assert np.allclose(r["probs"], 1e-3, rtol=1e-6)


def test_batch_independence_and_permutation(r18):
    ops, w, b = r18
    x = gen.images(0, 0, 4, 3, 64, 64, "uniform")
    whole = N.forward(ops, w, b, x, threads=1)["logits"]
    for i in range(4):
        assert np.array_equal(N.forward(ops, w, b, x[i:i + 1])["logits"][0], whole[i])
    perm = [2, 0, 3, 1]
    assert np.array_equal(N.forward(ops, w, b, x[perm], threads=2)["logits"], whole[perm])


def test_f32_and_f64_builds_agree(r18):
    ops, w, b = r18
    x = gen.images(0, 0, 1, 3, 64, 64, "uniform")
    z32 = N.forward(ops, w, b, x, prec="f32")["logits"]
    z64 = N.forward(ops, w, b, x, prec="f64")["logits"]
    assert np.abs(z32 - z64).max() <= 1e-5 * np.abs(z64).max()


def test_keep_all_returns_every_op_output(r18):
    ops, w, b = r18
    x = gen.images(0, 0, 1, 3, 64, 64, "uniform")
    outs = N.forward(ops, w, b, x, keep="all")
    assert len(outs) == len(ops)
    for o, (c, h, wd) in zip(outs[:-3], T.shapes(ops, 64, 64)[:-3]):
        assert o.shape == (1, c, h, wd)
    assert np.array_equal(outs[-2], N.forward(ops, w, b, x)["logits"])
    # post-ReLU outputs are non-negative, the projection shortcut's are not
    proj = [i for i, o in enumerate(ops) if o.op == T.CONV and not o.relu]
    assert proj and all((outs[i] < 0).any() for i in proj)
    assert all((outs[i] >= 0).all() for i, o in enumerate(ops) if o.op == T.CONV and o.relu)


def test_storage_mode_rounds_only_conv_outputs(r18):
    """The 16-bit-storage mode: conv outputs become exactly representable in that type,
    and the result stays within the type's rounding error of the definition."""
    ops, w, b = r18
    x = gen.images(0, 0, 1, 3, 64, 64, "uniform")
    plain = N.forward(ops, w, b, x, keep="all")
    for st, eps in (("fp16", 2.0 ** -11), ("bf16", 2.0 ** -8)):
        outs = N.forward(ops, w, b, x, keep="all", storage=st)
        for o, y in zip(ops, outs):
            if o.op in (T.CONV, T.MAXPOOL):
                assert np.array_equal(gen.quantize(y, st), y)
        # first conv: exactly the rounded plain result
        assert np.array_equal(outs[0], gen.quantize(plain[0], st))
        z, zp = outs[-2], plain[-2]
        assert 0 < np.abs(z - zp).max() <= 40 * eps * np.abs(zp).max()
