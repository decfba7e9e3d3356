"""Seeded, counter-based synthetic tensors (weights, biases, images).

This module only *draws numbers and lays bytes out*; it holds none of the
forward pass's arithmetic, so both the CPU oracle's tests and the HIP harness
may use it.  Every value is a pure function of (seed, stream, index):

    z   = key + (index + 1) * 0x9E3779B97F4A7C15          (mod 2^64)
    z   = splitmix64 finaliser(z)
    u   = (z >> 11) * 2^-53                                in [0, 1)
    key = splitmix64 finaliser(seed * 0xD1342543DE82EF95 + stream + 1)

Normals use Box-Muller on the counter pair (2i, 2i+1):
    n_i = sqrt(-2 ln(1 - u_{2i})) * cos(2 pi u_{2i+1}).

Recipes (paper Table 1 fixes only sizes: fp32 input of 3x224x224, 1000 fp32
outputs, weight blob sizes; the value distributions are this build's workload
definition):
  * conv / FC weights ~ N(0, 2 / fan_in), fan_in = cin*kh*kw, rounded once to
    the storage type (fp16 or bf16) with round-to-nearest-even;
  * biases (the folded BatchNorm shift) ~ N(0, 0.01) i.e. std 0.1, kept fp32;
  * images ~ N(0, 1) or U[-1, 1), rounded once to the storage type so that
    both consumers start from bit-identical values.

Canonical weight blob (what LOAD receives): for each op that owns weights, in
op order, W[cout][cin][kh][kw] in the storage type, all of them back to back;
then, after padding to a multiple of 4 bytes, every bias[cout] as fp32 in the
same op order.
"""
import numpy as np

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_KEYMUL = 0xD1342543DE82EF95
_MASK = (1 << 64) - 1

BIAS_STD = 0.1  # variance 0.01


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _key(seed, stream):
    k = (int(seed) * _KEYMUL + int(stream) + 1) & _MASK
    with np.errstate(over="ignore"):
        return _mix(np.array([k], dtype=np.uint64))[0]


def uniform01(seed, stream, n, offset=0):
    """n uniforms in [0,1), float64, counters offset .. offset+n-1."""
    with np.errstate(over="ignore"):
        idx = np.arange(offset + 1, offset + n + 1, dtype=np.uint64)
        z = _mix(_key(seed, stream) + idx * _GOLD)
    return (z >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def normal(seed, stream, n):
    """n standard normals, float64."""
    u = uniform01(seed, stream, 2 * n)
    return np.sqrt(-2.0 * np.log1p(-u[0::2])) * np.cos(2.0 * np.pi * u[1::2])


def round_bf16(x32):
    """float32 -> nearest-even bfloat16, returned as the uint16 bit pattern."""
    b = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_f32(bits16):
    return (bits16.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage_bits(x, dtype):
    """Round float values to the storage type; returns uint16 bit patterns."""
    x32 = np.asarray(x, dtype=np.float32)
    if dtype == "fp16":
        return x32.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        return round_bf16(x32)
    raise ValueError(dtype)


def from_storage_bits(bits, dtype):
    if dtype == "fp16":
        return bits.view(np.float16).astype(np.float32)
    if dtype == "bf16":
        return bf16_to_f32(bits)
    raise ValueError(dtype)


def quantize(x, dtype):
    """Round to the storage type and come back to float32 (exactly representable)."""
    return from_storage_bits(to_storage_bits(x, dtype), dtype)


def model_tensors(shapes, seed, dtype="fp16", weight_gain=None):
    """Weights and biases of a model.

    shapes: list of (cout, cin, kh, kw) in op order.
    weight_gain: optional list of per-tensor multipliers on the He std.
    Returns (weights, biases): float32 arrays; weights exactly representable in
    ``dtype``.  Tensor t draws weights from stream 2t and biases from 2t+1.
    """
    weights, biases = [], []
    for t, (k, c, r, s) in enumerate(shapes):
        std = np.sqrt(2.0 / (c * r * s))
        if weight_gain is not None:
            std *= weight_gain[t]
        w = normal(seed, 2 * t, k * c * r * s) * std
        weights.append(quantize(w.astype(np.float32), dtype).reshape(k, c, r, s))
        biases.append((normal(seed, 2 * t + 1, k) * BIAS_STD).astype(np.float32))
    return weights, biases


def pack_blob(weights, biases, dtype="fp16"):
    """Canonical LOAD blob (layout in the module docstring) as a uint8 array."""
    wbits = np.concatenate([to_storage_bits(w.ravel(), dtype) for w in weights])
    wbytes = wbits.view(np.uint8)
    padn = (-wbytes.size) % 4
    bbytes = np.concatenate([np.asarray(b, np.float32).ravel() for b in biases]).view(np.uint8)
    return np.concatenate([wbytes, np.zeros(padn, np.uint8), bbytes])


def blob_bytes(shapes, elem_bytes=2):
    nw = sum(k * c * r * s for (k, c, r, s) in shapes) * elem_bytes
    nw += (-nw) % 4
    return nw + 4 * sum(k for (k, _, _, _) in shapes)


IMAGE_STREAM = 1 << 20


def images(seed, first, count, c, h, w, dist="normal", dtype="fp16"):
    """Images first .. first+count-1 of the image set ``seed``: [count][c][h][w]
    float32, exactly representable in ``dtype``.  Image i has its own stream, so
    it does not depend on how the set is cut into batches."""
    out = np.empty((count, c, h, w), dtype=np.float32)
    n = c * h * w
    for i in range(count):
        st = IMAGE_STREAM + first + i
        if dist == "normal":
            v = normal(seed, st, n)
        elif dist == "uniform":
            v = uniform01(seed, st, n) * 2.0 - 1.0
        else:
            raise ValueError(dist)
        out[i] = quantize(v.astype(np.float32), dtype).reshape(c, h, w)
    return out
