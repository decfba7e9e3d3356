"""Python face of the C oracle: per-operator calls and the forward pass of an
operator list (test infrastructure; see the header of oracle.c).

``forward`` walks the list in order and applies, per op, exactly the steps the
definition states: conv (+bias), then the shortcut addition if the op has one,
then ReLU if the op has one.  Samples are independent, so a batch may be spread
over threads one sample each; the loops inside an operator are never touched.
"""
import ctypes
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from . import build as _build
from .topology import CONCAT, CONV, FC, GAVGPOOL, MAXPOOL, SOFTMAX, conv_geometry

_LIBS = {}


def _lib(prec):
    if prec not in _LIBS:
        _build.build()
        lib = ctypes.CDLL(_build.LIBS[prec][0])
        for name in ("orc_conv2d", "orc_relu", "orc_add", "orc_maxpool2d",
                     "orc_global_avgpool", "orc_fc", "orc_softmax", "orc_argmax",
                     "orc_conv2d_grouped", "orc_hswish", "orc_concat_channels"):
            getattr(lib, name).restype = None
        _LIBS[prec] = lib
    return _LIBS[prec]


def _dt(prec):
    return np.float32 if prec == "f32" else np.float64


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _arr(a, prec):
    return np.ascontiguousarray(a, dtype=_dt(prec))


def conv2d(x, w, b, stride, pad, prec="f32"):
    x, w = _arr(x, prec), _arr(w, prec)
    b = _arr(b, prec) if b is not None else None
    n, c, h, wd = x.shape
    k, c2, kh, kw = w.shape
    assert c == c2
    ho = (h + 2 * pad - kh) // stride + 1
    wo = (wd + 2 * pad - kw) // stride + 1
    y = np.empty((n, k, ho, wo), dtype=_dt(prec))
    _lib(prec).orc_conv2d(_p(x), _p(w), _p(b), _p(y), n, c, h, wd, k, kh, kw, stride, pad)
    return y


def conv2d_grouped(x, w, b, stride, pad_h, pad_w, groups, prec="f32"):
    """Grouped convolution, rectangular filter, separate paddings; w is [K][C/groups][kh][kw]."""
    x, w = _arr(x, prec), _arr(w, prec)
    b = _arr(b, prec) if b is not None else None
    n, c, h, wd = x.shape
    k, cg, kh, kw = w.shape
    assert c % groups == 0 and k % groups == 0 and cg == c // groups
    ho = (h + 2 * pad_h - kh) // stride + 1
    wo = (wd + 2 * pad_w - kw) // stride + 1
    y = np.empty((n, k, ho, wo), dtype=_dt(prec))
    _lib(prec).orc_conv2d_grouped(_p(x), _p(w), _p(b), _p(y), n, c, h, wd, k, kh, kw, stride, pad_h, pad_w, groups)
    return y


def hswish(x, prec="f32"):
    x = _arr(x, prec)
    y = np.empty_like(x)
    _lib(prec).orc_hswish(_p(x), _p(y), ctypes.c_size_t(x.size))
    return y


def concat_channels(a, b, prec="f32"):
    a, b = _arr(a, prec), _arr(b, prec)
    assert a.shape[0] == b.shape[0] and a.shape[2:] == b.shape[2:]
    n, ca = a.shape[:2]
    cb = b.shape[1]
    hw = int(np.prod(a.shape[2:]))
    y = np.empty((n, ca + cb) + a.shape[2:], dtype=_dt(prec))
    _lib(prec).orc_concat_channels(_p(a), _p(b), _p(y), n, ca, cb, hw)
    return y


def relu(x, prec="f32"):
    x = _arr(x, prec)
    y = np.empty_like(x)
    _lib(prec).orc_relu(_p(x), _p(y), ctypes.c_size_t(x.size))
    return y


def add(a, b, prec="f32"):
    a, b = _arr(a, prec), _arr(b, prec)
    assert a.shape == b.shape
    y = np.empty_like(a)
    _lib(prec).orc_add(_p(a), _p(b), _p(y), ctypes.c_size_t(a.size))
    return y


def maxpool2d(x, k, stride, pad, prec="f32"):
    x = _arr(x, prec)
    n, c, h, w = x.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    y = np.empty((n, c, ho, wo), dtype=_dt(prec))
    _lib(prec).orc_maxpool2d(_p(x), _p(y), n, c, h, w, k, k, stride, pad)
    return y


def global_avgpool(x, prec="f32"):
    x = _arr(x, prec)
    n, c, h, w = x.shape
    y = np.empty((n, c), dtype=_dt(prec))
    _lib(prec).orc_global_avgpool(_p(x), _p(y), n, c, h, w)
    return y


def fc(f, w, b, prec="f32"):
    f, w = _arr(f, prec), _arr(w, prec)
    b = _arr(b, prec) if b is not None else None
    n, i = f.shape
    o, i2 = w.shape
    assert i == i2
    z = np.empty((n, o), dtype=_dt(prec))
    _lib(prec).orc_fc(_p(f), _p(w), _p(b), _p(z), n, i, o)
    return z


def softmax(z, prec="f32"):
    z = _arr(z, prec)
    n, d = z.shape
    p = np.empty_like(z)
    _lib(prec).orc_softmax(_p(z), _p(p), n, d)
    return p


def argmax(z, prec="f32"):
    z = _arr(z, prec)
    n, d = z.shape
    idx = np.empty(n, dtype=np.int32)
    _lib(prec).orc_argmax(_p(z), _p(idx), n, d)
    return idx


def _round_storage(y, storage):
    """Round every element once (nearest even) to a 16-bit storage type and return
    to the working precision.  Models a path that keeps activations in that type
    between operators; the arithmetic inside an operator is unchanged."""
    if storage is None:
        return y
    y32 = y.astype(np.float32)
    if storage == "fp16":
        q = y32.astype(np.float16).astype(np.float32)
    elif storage == "bf16":
        b = y32.view(np.uint32)
        r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
        q = r.view(np.float32)
    else:
        raise ValueError(storage)
    return q.astype(y.dtype)


def _forward_one(ops, weights, biases, x, prec, keep, storage=None):
    """Forward pass of a batch held in one array; returns dict of kept outputs."""
    outs = []
    wi = 0
    for o in ops:
        src = x if o.input_from < 0 else outs[o.input_from]
        if o.op == CONV:
            pad_h, pad_w, groups = conv_geometry(o)
            if groups == 1 and o.kh == o.kw:
                y = conv2d(src, weights[wi], biases[wi], o.stride, o.pad, prec)
            else:
                y = conv2d_grouped(src, weights[wi], biases[wi], o.stride, pad_h, pad_w, groups, prec)
            wi += 1
            if o.residual_from >= 0:
                y = add(y, outs[o.residual_from], prec)
            if o.relu == 1:
                y = relu(y, prec)
            elif o.relu == 2:
                y = hswish(y, prec)
            y = _round_storage(y, storage)
        elif o.op == CONCAT:
            y = concat_channels(src, outs[o.residual_from], prec)
        elif o.op == MAXPOOL:
            y = maxpool2d(src, o.kh, o.stride, o.pad, prec)
        elif o.op == GAVGPOOL:
            y = global_avgpool(src, prec)
        elif o.op == FC:
            y = fc(src.reshape(src.shape[0], -1), weights[wi].reshape(o.cout, o.cin),
                   biases[wi], prec)
            wi += 1
        elif o.op == SOFTMAX:
            y = softmax(src, prec)
        else:
            raise ValueError("unknown op %r" % (o.op,))
        outs.append(y)
    if keep == "all":
        return outs
    res = {}
    for i, o in enumerate(ops):
        if o.op == FC:
            res["logits"] = outs[i]
        elif o.op == SOFTMAX:
            res["probs"] = outs[i]
    return res


def forward(ops, weights, biases, x, prec="f32", threads=None, keep="final", storage=None):
    """EXEC of one batch.  ``weights[i]``/``biases[i]`` belong to the i-th op that
    owns weights (conv or FC, in op order); ``x`` is [N][C][H][W].

    storage=None is the definition itself.  storage="fp16"/"bf16" is a second mode
    that rounds each convolution's final output (after bias, shortcut and ReLU) once
    to that type, as a path storing its feature maps in 16 bits does; pooled
    features, logits and probabilities stay in the working precision.

    keep="final": returns {"logits": [N][classes], "probs": [N][classes]}.
    keep="all":   returns the list of every op's output (NCHW), whole batch,
                  computed in the calling thread.
    """
    x = _arr(x, prec)
    if keep == "all":
        return _forward_one(ops, weights, biases, x, prec, "all", storage)
    n = x.shape[0]
    threads = threads or min(n, len(os.sched_getaffinity(0)))
    if threads <= 1 or n == 1:
        return _forward_one(ops, weights, biases, x, prec, "final", storage)
    with ThreadPoolExecutor(max_workers=threads) as ex:
        parts = list(ex.map(
            lambda i: _forward_one(ops, weights, biases, x[i:i + 1], prec, "final", storage),
            range(n)))
    return {k: np.concatenate([p[k] for p in parts], axis=0) for k in parts[0]}
