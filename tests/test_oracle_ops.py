"""Pins for the CPU oracle's operators (no GPU): brute force, closed forms,
special cases that reduce to library routines.  Each pin is chosen so that a
plausible slip in oracle.c (dropped term, wrong sign/index, transposed operand,
kernel flip, wrong padding rule) fails at least one of them."""
import itertools

import numpy as np
import pytest
import torch

from oracle import network as N

RNG = np.random.default_rng(1234)


def gather_conv(x, w, b, st, pad):
    """Independent float64 definition, gather style: build each output element's
    receptive field (zero padded) and dot it with the filter."""
    n, c, h, wd = x.shape
    k, _, kh, kw = w.shape
    xp = np.zeros((n, c, h + 2 * pad, wd + 2 * pad))
    xp[:, :, pad:pad + h, pad:pad + wd] = x
    ho = (h + 2 * pad - kh) // st + 1
    wo = (wd + 2 * pad - kw) // st + 1
    y = np.empty((n, k, ho, wo))
    for i, j, p, q in itertools.product(range(n), range(k), range(ho), range(wo)):
        patch = xp[i, :, p * st:p * st + kh, q * st:q * st + kw]
        y[i, j, p, q] = np.dot(patch.ravel(), w[j].ravel()) + b[j]
    return y


CONV_CASES = [
    # n c h w k kh st pad
    (1, 1, 5, 5, 1, 1, 1, 0),
    (2, 3, 7, 6, 4, 3, 1, 1),
    (2, 5, 9, 8, 3, 3, 2, 1),
    (1, 3, 9, 9, 2, 7, 2, 3),
    (1, 4, 8, 8, 3, 1, 2, 0),
    (2, 2, 6, 9, 2, 3, 1, 0),
    (1, 2, 7, 7, 2, 7, 1, 3),
]


@pytest.mark.parametrize("case", CONV_CASES)
@pytest.mark.parametrize("prec,tol", [("f32", 2e-6), ("f64", 1e-13)])
def test_conv_brute_force(case, prec, tol):
    n, c, h, w, k, kk, st, pad = case
    x = RNG.standard_normal((n, c, h, w))
    wt = RNG.standard_normal((k, c, kk, kk))
    b = RNG.standard_normal(k)
    ref = gather_conv(x, wt, b, st, pad)
    got = N.conv2d(x, wt, b, st, pad, prec)
    assert got.shape == ref.shape
    assert np.abs(got - ref).max() <= tol * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_vs_torch_f64(case):
    n, c, h, w, k, kk, st, pad = case
    x = RNG.standard_normal((n, c, h, w))
    wt = RNG.standard_normal((k, c, kk, kk))
    b = RNG.standard_normal(k)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(wt),
                                     torch.from_numpy(b), stride=st, padding=pad).numpy()
    got = N.conv2d(x, wt, b, st, pad, "f64")
    assert np.abs(got - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())


def test_conv_identity_kernel_returns_input_plus_bias():
    c = 5
    x = RNG.standard_normal((2, c, 6, 7)).astype(np.float32)
    w = np.eye(c, dtype=np.float32).reshape(c, c, 1, 1)
    b = np.arange(c, dtype=np.float32)
    y = N.conv2d(x, w, b, 1, 0)
    assert np.array_equal(y, x + b.reshape(1, c, 1, 1))


@pytest.mark.parametrize("r,s", [(0, 0), (0, 2), (2, 1), (1, 1), (2, 2)])
@pytest.mark.parametrize("st", [1, 2])
def test_conv_delta_kernel_shifts_without_flip(r, s, st):
    """A single 1 at filter tap (r, s) must give y[p][q] = x[p*st-1+r][q*st-1+s]
    (zero outside): cross-correlation, not flipped convolution."""
    h, wd = 7, 8
    x = RNG.standard_normal((1, 1, h, wd)).astype(np.float32)
    w = np.zeros((1, 1, 3, 3), np.float32)
    w[0, 0, r, s] = 1.0
    y = N.conv2d(x, w, None, st, 1)
    ho, wo = (h + 2 - 3) // st + 1, (wd + 2 - 3) // st + 1
    assert y.shape == (1, 1, ho, wo)
    for p in range(ho):
        for q in range(wo):
            ih, iw = p * st - 1 + r, q * st - 1 + s
            exp = x[0, 0, ih, iw] if (0 <= ih < h and 0 <= iw < wd) else 0.0
            assert y[0, 0, p, q] == exp


@pytest.mark.parametrize("kk,st,pad", [(3, 1, 1), (3, 2, 1), (7, 2, 3), (1, 1, 0)])
def test_conv_constant_closed_form(kk, st, pad):
    """Constant input c0, constant weight w0: y = c0*w0*Cin*(#in-range taps) + b."""
    c0, w0, cin, h, wd = 0.5, 0.25, 4, 9, 10
    x = np.full((1, cin, h, wd), c0, np.float32)
    w = np.full((2, cin, kk, kk), w0, np.float32)
    b = np.array([1.0, -2.0], np.float32)
    y = N.conv2d(x, w, b, st, pad)
    ho, wo = y.shape[2:]
    for p in range(ho):
        for q in range(wo):
            rows = sum(0 <= p * st - pad + r < h for r in range(kk))
            cols = sum(0 <= q * st - pad + s < wd for s in range(kk))
            for k in range(2):
                assert y[0, k, p, q] == c0 * w0 * cin * rows * cols + b[k]
    # interior check: full window
    if kk > 1:
        assert y[0, 0, ho // 2, wo // 2] == c0 * w0 * cin * kk * kk + b[0]


def test_conv_1x1_is_matrix_product():
    n, c, h, wd, k = 2, 16, 5, 6, 7
    x = RNG.standard_normal((n, c, h, wd))
    w = RNG.standard_normal((k, c, 1, 1))
    b = RNG.standard_normal(k)
    got = N.conv2d(x, w, b, 1, 0, "f64")
    xm = x.transpose(0, 2, 3, 1).reshape(-1, c)            # [M][C]
    ym = xm @ w.reshape(k, c).T + b                          # [M][K]
    ref = ym.reshape(n, h, wd, k).transpose(0, 3, 1, 2)
    assert np.abs(got - ref).max() < 1e-12


def test_conv_1x1_stride2_subsamples():
    x = RNG.standard_normal((1, 3, 8, 8)).astype(np.float32)
    w = RNG.standard_normal((4, 3, 1, 1)).astype(np.float32)
    full = N.conv2d(x, w, None, 1, 0)
    sub = N.conv2d(x, w, None, 2, 0)
    assert np.array_equal(sub, full[:, :, ::2, ::2])


def test_relu_and_add():
    a = np.array([-1.5, 0.0, 2.0, -0.0, 3.5], np.float32)
    assert np.array_equal(N.relu(a), np.array([0, 0, 2.0, 0, 3.5], np.float32))
    b = np.array([1.0, 2.0, -2.0, 4.0, 0.5], np.float32)
    assert np.array_equal(N.add(a, b), a + b)


def test_maxpool_ramp_closed_form():
    """x[h][w] = h*W + w is increasing in both axes, so each window's max is its
    last in-range element."""
    h, wd = 9, 11
    x = np.arange(h * wd, dtype=np.float32).reshape(1, 1, h, wd)
    y = N.maxpool2d(x, 3, 2, 1)
    ho, wo = (h + 2 - 3) // 2 + 1, (wd + 2 - 3) // 2 + 1
    assert y.shape == (1, 1, ho, wo)
    for p in range(ho):
        for q in range(wo):
            ih = min(2 * p - 1 + 2, h - 1)
            iw = min(2 * q - 1 + 2, wd - 1)
            assert y[0, 0, p, q] == ih * wd + iw


def test_maxpool_ignores_padding_for_negative_input():
    x = -np.ones((1, 2, 6, 6), np.float32) - RNG.random((1, 2, 6, 6)).astype(np.float32)
    y = N.maxpool2d(x, 3, 2, 1)
    assert (y < 0).all()          # zero padding would have produced 0 at the border
    ref = torch.nn.functional.max_pool2d(torch.from_numpy(x), 3, 2, 1).numpy()
    assert np.array_equal(y, ref)


def test_maxpool_zero_pad_equivalent_for_nonnegative_input():
    x = RNG.random((2, 3, 8, 8)).astype(np.float32)
    xp = np.zeros((2, 3, 10, 10), np.float32)
    xp[:, :, 1:9, 1:9] = x
    assert np.array_equal(N.maxpool2d(x, 3, 2, 1), N.maxpool2d(xp, 3, 2, 0))


def test_global_avgpool():
    x = RNG.standard_normal((3, 4, 5, 7))
    assert np.abs(N.global_avgpool(x, "f64") - x.mean(axis=(2, 3))).max() < 1e-14
    c = np.full((1, 2, 7, 7), 3.25, np.float32)
    assert np.array_equal(N.global_avgpool(c), np.full((1, 2), 3.25, np.float32))


def test_fc_matches_matmul_and_is_not_transposed():
    f = RNG.standard_normal((3, 11))
    w = RNG.standard_normal((5, 11))
    b = RNG.standard_normal(5)
    assert np.abs(N.fc(f, w, b, "f64") - (f @ w.T + b)).max() < 1e-13
    # one-hot feature i picks column i of W: z[j] = W[j][i] + b[j]
    e = np.zeros((1, 11)); e[0, 4] = 1.0
    assert np.allclose(N.fc(e, w, b, "f64")[0], w[:, 4] + b, atol=0, rtol=0)


def test_softmax_properties():
    z = RNG.standard_normal((4, 1000)) * 3
    p = N.softmax(z, "f64")
    assert np.abs(p.sum(1) - 1).max() < 1e-12
    assert np.abs(N.softmax(z + 123.0, "f64") - p).max() < 1e-12      # shift invariance
    u = N.softmax(np.zeros((1, 1000), np.float32))
    assert np.allclose(u, 1e-3, rtol=1e-6)
    import scipy.special
    assert np.abs(p - scipy.special.softmax(z, axis=1)).max() < 1e-14
    # two classes: softmax = logistic of the difference
    z2 = np.array([[0.3, -1.1]])
    assert abs(N.softmax(z2, "f64")[0, 0] - 1 / (1 + np.exp(-1.4))) < 1e-15
    # huge logits do not overflow
    big = np.array([[5000.0, 4000.0, -3000.0]], np.float32)
    assert np.array_equal(N.softmax(big), np.array([[1, 0, 0]], np.float32))
    p32 = N.softmax(z.astype(np.float32))
    assert np.abs(p32.sum(1) - 1).max() < 1e-5


def test_argmax_ties_and_scale_invariance():
    z = np.array([[1, 7, 7, 3], [2, 2, 2, 2], [-1, -5, -1, -9]], np.float32)
    assert list(N.argmax(z)) == [1, 0, 0]
    r = RNG.standard_normal((16, 1000)).astype(np.float32)
    base = N.argmax(r)
    assert np.array_equal(base, np.argmax(r, axis=1))
    for a in (0.5, 3.0, 1e-3, 1e4):
        assert np.array_equal(N.argmax(r * np.float32(a)), base)
