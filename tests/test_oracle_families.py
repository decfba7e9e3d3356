"""Pins for the oracle's operators of the other model families (grouped / depthwise / rectangular
convolution, hard swish, channel concatenation) and for the operator lists built from them.  No GPU.
Each pin is something other than the oracle's own formula: a gather-style float64 brute force, a
library routine, a closed form, or a reduction to the dense square convolution that
test_oracle_ops.py already pins."""
import itertools

import numpy as np
import pytest
import torch

from oracle import network as N
from oracle import topology as T

RNG = np.random.default_rng(4321)


def gather_grouped(x, w, b, st, ph, pw, groups):
    """float64, gather style: every output element's receptive field inside its own channel group."""
    n, c, h, wd = x.shape
    k, cg, kh, kw = w.shape
    kg = k // groups
    xp = np.zeros((n, c, h + 2 * ph, wd + 2 * pw))
    xp[:, :, ph:ph + h, pw:pw + wd] = x
    ho = (h + 2 * ph - kh) // st + 1
    wo = (wd + 2 * pw - kw) // st + 1
    y = np.empty((n, k, ho, wo))
    for i, j, p, q in itertools.product(range(n), range(k), range(ho), range(wo)):
        g = j // kg
        patch = xp[i, g * cg:(g + 1) * cg, p * st:p * st + kh, q * st:q * st + kw]
        y[i, j, p, q] = np.dot(patch.ravel(), w[j].ravel()) + b[j]
    return y


GROUPED_CASES = [
    # n  c  h  w   k kh kw st ph pw groups
    (2,  4, 7, 6,  4, 3, 3, 1, 1, 1, 4),     # depthwise 3x3
    (1,  6, 9, 8,  6, 3, 3, 2, 1, 1, 6),     # depthwise stride 2
    (2,  6, 5, 7,  4, 3, 3, 1, 1, 1, 2),     # two groups, K != C
    (1,  3, 6, 9,  2, 1, 7, 1, 0, 3, 1),     # 1x7, padding only in width
    (1,  3, 9, 6,  2, 7, 1, 1, 3, 0, 1),     # 7x1, padding only in height
    (2,  2, 8, 8,  3, 3, 5, 2, 0, 2, 1),     # rectangular, strided, mixed padding
    (1,  4, 6, 6,  4, 5, 5, 1, 2, 2, 4),     # depthwise 5x5
]


@pytest.mark.parametrize("case", GROUPED_CASES)
@pytest.mark.parametrize("prec,tol", [("f32", 2e-6), ("f64", 1e-13)])
def test_grouped_conv_brute_force(case, prec, tol):
    n, c, h, w, k, kh, kw, st, ph, pw, g = case
    x = RNG.standard_normal((n, c, h, w))
    wt = RNG.standard_normal((k, c // g, kh, kw))
    b = RNG.standard_normal(k)
    ref = gather_grouped(x, wt, b, st, ph, pw, g)
    got = N.conv2d_grouped(x, wt, b, st, ph, pw, g, prec)
    assert got.shape == ref.shape
    assert np.abs(got - ref).max() <= tol * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("case", GROUPED_CASES)
def test_grouped_conv_vs_torch_f64(case):
    n, c, h, w, k, kh, kw, st, ph, pw, g = case
    x = RNG.standard_normal((n, c, h, w))
    wt = RNG.standard_normal((k, c // g, kh, kw))
    b = RNG.standard_normal(k)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(wt), torch.from_numpy(b),
                                     stride=st, padding=(ph, pw), groups=g).numpy()
    got = N.conv2d_grouped(x, wt, b, st, ph, pw, g, "f64")
    assert np.abs(got - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())


def test_grouped_conv_is_the_dense_conv_per_group():
    """A grouped convolution is the dense one (pinned on its own) applied to each channel group."""
    x = RNG.standard_normal((2, 6, 7, 7))
    wt = RNG.standard_normal((9, 2, 3, 3))
    b = RNG.standard_normal(9)
    got = N.conv2d_grouped(x, wt, b, 1, 1, 1, 3, "f64")
    for g in range(3):
        part = N.conv2d(x[:, 2 * g:2 * g + 2], wt[3 * g:3 * g + 3], b[3 * g:3 * g + 3], 1, 1, "f64")
        assert np.array_equal(got[:, 3 * g:3 * g + 3], part)
    # and with one group and a square filter it is the dense convolution itself
    assert np.array_equal(N.conv2d_grouped(x, RNG.integers(-2, 3, (4, 6, 3, 3)).astype(float), None, 2, 1, 1, 1, "f64").shape,
                          (2, 4, 4, 4))
    w1 = RNG.standard_normal((4, 6, 3, 3))
    assert np.array_equal(N.conv2d_grouped(x, w1, None, 2, 1, 1, 1, "f64"), N.conv2d(x, w1, None, 2, 1, "f64"))


def test_depthwise_delta_shifts_each_channel_on_its_own():
    """A depthwise filter with a single 1 at (r, s), different per channel, returns each channel
    shifted by its own offset and zero padded: no channel may leak into another."""
    c, h, w = 3, 6, 7
    x = RNG.integers(-5, 6, (1, c, h, w)).astype(np.float32)
    taps = [(0, 0), (1, 2), (2, 1)]
    wt = np.zeros((c, 1, 3, 3), np.float32)
    for ch, (r, s) in enumerate(taps):
        wt[ch, 0, r, s] = 1
    y = N.conv2d_grouped(x, wt, None, 1, 1, 1, c)
    xp = np.zeros((c, h + 2, w + 2), np.float32)
    xp[:, 1:-1, 1:-1] = x[0]
    for ch, (r, s) in enumerate(taps):
        assert np.array_equal(y[0, ch], xp[ch, r:r + h, s:s + w])


def test_1x7_then_7x1_is_the_7x7_with_the_outer_product_filter():
    """Zero padding commutes with the two passes, so a 1x7 convolution (padding 0, 3) followed by a
    7x1 convolution (padding 3, 0) equals the 7x7 convolution (padding 3) whose filter is the outer
    product of the two; small integers make every sum exact in fp32."""
    x = RNG.integers(-3, 4, (1, 1, 9, 10)).astype(np.float32)
    a = RNG.integers(-2, 3, 7).astype(np.float32)      # along the width
    b = RNG.integers(-2, 3, 7).astype(np.float32)      # along the height
    z = N.conv2d_grouped(x, a.reshape(1, 1, 1, 7), None, 1, 0, 3, 1)
    y = N.conv2d_grouped(z, b.reshape(1, 1, 7, 1), None, 1, 3, 0, 1)
    full = N.conv2d(x, np.outer(b, a).reshape(1, 1, 7, 7), None, 1, 3)
    assert np.array_equal(y, full)
    # a transposed operand (7x1 where 1x7 was meant) changes the output shape or values
    zt = N.conv2d_grouped(x, a.reshape(1, 1, 7, 1), None, 1, 3, 0, 1)
    assert not np.array_equal(zt, z)


def test_constant_input_border_tap_counts_rectangular():
    """Constant input c, constant filter w, no bias: every output is c * w * (taps inside the image)."""
    h, wd, kh, kw, ph, pw = 5, 6, 3, 5, 1, 2
    x = np.full((1, 2, h, wd), 2.0, np.float32)
    wt = np.full((1, 2, kh, kw), 0.5, np.float32)
    y = N.conv2d_grouped(x, wt, None, 1, ph, pw, 1)[0, 0]
    for p in range(h):
        for q in range(wd):
            rows = sum(0 <= p - ph + r < h for r in range(kh))
            cols = sum(0 <= q - pw + s < wd for s in range(kw))
            assert y[p, q] == 2.0 * 0.5 * 2 * rows * cols


def test_hswish_closed_form_points():
    x = np.array([-5.0, -3.0, -1.5, -1.0, 0.0, 1.0, 3.0, 4.5], np.float64)
    want = np.array([0.0, 0.0, -0.375, -1.0 / 3.0, 0.0, 4.0 / 6.0, 3.0, 4.5])
    assert np.allclose(N.hswish(x, "f64"), want, rtol=0, atol=1e-15)
    y32 = N.hswish(x.astype(np.float32))
    assert np.abs(y32 - want).max() <= 1e-6
    # library routine in float64
    big = RNG.standard_normal(1000) * 4
    assert np.abs(N.hswish(big, "f64") - torch.nn.functional.hardswish(torch.from_numpy(big)).numpy()).max() <= 1e-15
    # identity above 3, zero below -3, minimum -3/8 at -3/2
    assert N.hswish(big, "f64").min() >= -0.375


def test_concat_keeps_both_blocks_in_order():
    a = RNG.standard_normal((2, 3, 4, 5)).astype(np.float32)
    b = RNG.standard_normal((2, 2, 4, 5)).astype(np.float32)
    y = N.concat_channels(a, b)
    assert y.shape == (2, 5, 4, 5)
    assert np.array_equal(y[:, :3], a) and np.array_equal(y[:, 3:], b)
    assert np.array_equal(y, np.concatenate([a, b], axis=1))


# ---------------------------------------------------------------- operator lists
def test_mobilenet_counts_match_the_published_ones():
    """The depthwise-separable stack at width 1.0 and 224x224 has the parameter and multiply-add
    counts its paper gives (4.2 million parameters, 569 million mult-adds)."""
    ops = T.mobilenet()
    assert T.param_count(ops) == 4_221_032
    assert T.mac_count(ops, 224, 224) == 568_740_352
    sh = T.shapes(ops, 224, 224)
    assert sh[0] == (32, 112, 112) and sh[-4] == (1024, 7, 7)
    dw = [o for o in ops if o.op == T.CONV and o.groups > 1]
    assert len(dw) == 13 and all(o.groups == o.cin == o.cout for o in dw)
    assert {o.relu for o in ops if o.op == T.CONV} == {1, 2}


def test_dense_and_inception_lists_are_consistent():
    for ops, hw in ((T.dense_net(), 224), (T.inception_net(), 128)):
        sh = T.shapes(ops, hw, hw)
        for o, (c, h, w) in zip(ops, sh):
            if o.op == T.CONCAT:
                a, b = sh[o.input_from], sh[o.residual_from]
                assert a[1:] == b[1:] == (h, w) and a[0] + b[0] == c == o.cout and a[0] == o.cin
            elif o.input_from >= 0:
                assert sh[o.input_from][0] == o.cin
            if o.op == T.CONV and o.residual_from >= 0:
                assert sh[o.residual_from] == (c, h, w)
    d = T.dense_net()
    assert sum(o.op == T.CONCAT for o in d) == 18 and T.shapes(d, 224, 224)[-4] == (512, 28, 28)


def _tiny_case(ops, hw, seed):
    from workload import gen
    w, b = gen.model_tensors(T.weight_shapes(ops), seed)
    x = gen.images(seed, 0, 2, 3, hw, hw, "uniform")
    return w, b, x


def test_forward_of_the_new_lists_against_torch_f64():
    """Whole forward pass of small instances of the three families against the same graph built from
    library routines in float64 (conv2d with groups / rectangular padding, hardswish, cat)."""
    F = torch.nn.functional
    for ops, hw in ((T.mobilenet(num_classes=10), 32), (T.dense_net(num_classes=10, layers=(2, 2)), 32),
                    (T.inception_net(num_classes=10, width=32, blocks=1), 32)):
        w, b, x = _tiny_case(ops, hw, 3)
        got = N.forward(ops, w, b, x, prec="f64", threads=1)["logits"]
        outs, wi = [], 0
        for o in ops:
            src = torch.from_numpy(x.astype(np.float64)) if o.input_from < 0 else outs[o.input_from]
            if o.op == T.CONV:
                ph, pw, g = T.conv_geometry(o)
                y = F.conv2d(src, torch.from_numpy(w[wi].astype(np.float64)), torch.from_numpy(b[wi].astype(np.float64)),
                             stride=o.stride, padding=(ph, pw), groups=g)
                wi += 1
                if o.residual_from >= 0:
                    y = y + outs[o.residual_from]
                y = F.relu(y) if o.relu == 1 else (F.hardswish(y) if o.relu == 2 else y)
            elif o.op == T.MAXPOOL:
                y = F.max_pool2d(src, o.kh, o.stride, o.pad)
            elif o.op == T.CONCAT:
                y = torch.cat([src, outs[o.residual_from]], dim=1)
            elif o.op == T.GAVGPOOL:
                y = src.mean(dim=(2, 3))
            elif o.op == T.FC:
                y = F.linear(src, torch.from_numpy(w[wi].reshape(o.cout, o.cin).astype(np.float64)), torch.from_numpy(b[wi].astype(np.float64)))
                wi += 1
            elif o.op == T.SOFTMAX:
                y = F.softmax(src, dim=1)
            outs.append(y)
        ref = outs[-2].numpy()
        assert np.abs(got - ref).max() <= 1e-10 * np.abs(ref).max()
