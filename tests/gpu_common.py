"""Helpers of the GPU parity tests: the same seeded tensors go to the oracle (as
float32 arrays) and to the library (as the canonical blob)."""
import numpy as np

from oracle import network as N
from oracle import topology as T
from workload import gen

TOL = 2e-2   # max |z_gpu - z_ref| / max |z_ref| per sample (spec tolerance)


class Case:
    def __init__(self, ops, in_hw, seed, dtype="fp16", dist="normal", weight_gain=None):
        self.ops = ops
        self.hw = in_hw
        self.seed = seed
        self.dtype = dtype
        self.dist = dist
        self.w, self.b = gen.model_tensors(T.weight_shapes(ops), seed, dtype, weight_gain)
        self.blob = gen.pack_blob(self.w, self.b, dtype)

    def images(self, first, count):
        return gen.images(self.seed, first, count, 3, self.hw, self.hw, self.dist, self.dtype)

    def oracle(self, x, keep="final", threads=None, storage=None):
        return N.forward(self.ops, self.w, self.b, x, prec="f32", threads=threads, keep=keep,
                         storage=storage)


def rel_err_per_sample(z_gpu, z_ref):
    """max_j |z_gpu - z_ref| / max_j |z_ref| for every sample."""
    return np.abs(z_gpu - z_ref).max(axis=1) / np.abs(z_ref).max(axis=1)


def top2_gap(z):
    s = np.sort(z, axis=1)
    return s[:, -1] - s[:, -2]
