"""ctypes binding of include/clockwork_exec.h: same names, argument marshalling
only.  Every step of the path runs in the library's HIP kernels."""
import ctypes
import os
from ctypes import (POINTER, Structure, byref, c_char, c_char_p, c_float, c_int32,
                    c_int64, c_size_t, c_uint32, c_uint64, c_void_p)

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libclockwork_exec.so")

CW_OK = 0
CW_ERR_INVALID, CW_ERR_HIP, CW_ERR_NO_MEMORY, CW_ERR_NOT_LOADED = -1, -2, -3, -4
CW_ERR_ALREADY_LOADED, CW_ERR_NO_INPUT, CW_ERR_BAD_BATCH, CW_ERR_BUSY = -5, -6, -7, -8
CW_ERR_UNSUPPORTED, CW_ERR_NO_SLOT, CW_ERR_TOO_LATE, CW_ERR_TIMEOUT = -9, -10, -11, -12
CW_OP_CONV, CW_OP_MAXPOOL, CW_OP_GAVGPOOL, CW_OP_FC, CW_OP_SOFTMAX, CW_OP_CONCAT = 0, 1, 2, 3, 4, 5
CW_DTYPE_FP16, CW_DTYPE_BF16 = 0, 1
DTYPES = {"fp16": CW_DTYPE_FP16, "bf16": CW_DTYPE_BF16}
CONV_TILES = {"128x128": 0, "128x64": 1, "64x64": 2, "64x32": 3, "32x64": 4, "32x32": 5,
              "128x64w2": 6, "64x128w2": 7, "256x64": 8, "128x128w8": 9,
              "128x64k128": 10, "64x64k128": 11, "64x32k128": 12, "32x64k128": 13, "32x32k128": 14,
              "128x64k128g2": 15, "64x64k128g2": 16, "64x64k128g4": 17, "64x32k128g4": 18, "32x64k128g4": 19,
              "32x32k128g4": 20, "32x32k128g8": 21, "128x64g2": 22, "64x64g2": 23, "32x32g4": 24,
              "256x128w8": 25, "128x256w8": 26, "256x256w8": 27, "256x128": 28}


class cw_op(Structure):
    _fields_ = [(n, c_int32) for n in ("op", "cin", "cout", "kh", "kw", "stride", "pad",
                                        "relu", "residual_from", "input_from", "pad_w", "groups")]


class cw_config(Structure):
    _fields_ = [("device", c_int32), ("workspace_bytes", c_size_t), ("io_bytes", c_size_t),
                ("weight_pool_bytes", c_size_t), ("load_staging_bytes", c_size_t), ("weight_page_bytes", c_size_t)]


class cw_profile(Structure):
    _fields_ = [("n", c_uint32), ("p50_us", c_float), ("p99_us", c_float), ("p999_us", c_float),
                ("min_us", c_float), ("max_us", c_float), ("mean_us", c_float), ("p9999_us", c_float)]


class cw_launch_info(Structure):
    _fields_ = [("op_index", c_int32), ("fused_op", c_int32), ("proj_op", c_int32), ("pair_op", c_int32), ("kind", c_int32), ("grid_x", c_int32), ("grid_y", c_int32),
                ("grid_z", c_int32), ("block", c_int32), ("tile_m", c_int32), ("tile_n", c_int32),
                ("tile_k", c_int32), ("split_k", c_int32), ("conv_tile", c_int32), ("wave_groups", c_int32), ("next_op", c_int32), ("panels", c_int32), ("gemm_m", c_int64), ("gemm_n", c_int64), ("gemm_k", c_int64),
                ("bytes", c_int64), ("flops", c_int64), ("name", c_char * 48)]


class cw_action(Structure):
    _fields_ = [("id", c_int64), ("type", c_int32), ("model_id", c_int32), ("batch", c_int32), ("earliest_ns", c_uint64),
                ("latest_ns", c_uint64), ("host_in", c_void_p), ("host_in_bytes", c_size_t), ("host_probs", c_void_p),
                ("host_logits", c_void_p)]


class cw_result(Structure):
    _fields_ = [("id", c_int64), ("type", c_int32), ("status", c_int32), ("begin_ns", c_uint64), ("end_ns", c_uint64),
                ("device_ns", c_uint64)]


CW_ACTION_LOAD, CW_ACTION_UNLOAD, CW_ACTION_INFER = 1, 2, 3

# name -> (restype, argtypes); every symbol the header declares
SIGNATURES = {
    "cw_create": (c_int32, [POINTER(c_void_p), POINTER(cw_config)]),
    "cw_destroy": (c_int32, [c_void_p]),
    "cw_model_define": (c_int32, [c_void_p, POINTER(cw_op), c_int32, c_int32, c_int32, c_int32,
                                  POINTER(c_int32), c_int32, c_int32, POINTER(c_int32)]),
    "cw_model_define_resnet": (c_int32, [c_void_p, c_int32, c_int32, c_int32, c_int32, POINTER(c_int32)]),
    "cw_model_get_ops": (c_int32, [c_void_p, c_int32, POINTER(cw_op), c_int32, POINTER(c_int32)]),
    "cw_model_weight_bytes": (c_size_t, [c_void_p, c_int32]),
    "cw_model_workspace_bytes": (c_size_t, [c_void_p, c_int32, c_int32]),
    "cw_load_weights": (c_int32, [c_void_p, c_int32, c_void_p, c_size_t, c_void_p]),
    "cw_load_weights_begin": (c_int32, [c_void_p, c_int32, c_void_p, c_size_t, c_void_p, POINTER(c_void_p)]),
    "cw_load_weights_record": (c_int32, [c_void_p, c_void_p]),
    "cw_load_weights_end": (c_int32, [c_void_p, c_void_p]),
    "cw_load_weights_release": (None, [c_void_p]),
    "cw_unload_weights": (c_int32, [c_void_p, c_int32]),
    "cw_weight_pool_free": (c_size_t, [c_void_p]),
    "cw_weight_pages_free": (c_int32, [c_void_p]),
    "cw_context_device": (c_int32, [c_void_p]),
    "cw_worker_create": (c_int32, [c_void_p, POINTER(c_int32), POINTER(c_void_p)]),
    "cw_worker_destroy": (c_int32, [c_void_p]),
    "cw_worker_now_ns": (c_uint64, []),
    "cw_worker_submit": (c_int32, [c_void_p, POINTER(cw_action)]),
    "cw_worker_next_result": (c_int32, [c_void_p, POINTER(cw_result), c_uint64]),
    "cw_worker_profile": (c_int32, [c_void_p, c_int32, c_int32, c_int32, POINTER(c_uint32), POINTER(c_uint64), POINTER(c_uint64)]),
    "cw_model_weight_pages": (c_int32, [c_void_p, c_int32]),
    "cw_input": (c_int32, [c_void_p, c_int32, c_int32, c_void_p, POINTER(c_int32), c_void_p]),
    "cw_exec": (c_int32, [c_void_p, c_int32, c_int32, c_int32, c_void_p]),
    "cw_exec_static": (c_int32, [c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p]),
    "cw_exec_static_capacity": (c_size_t, []),
    "cw_output": (c_int32, [c_void_p, c_int32, c_void_p, c_void_p, c_void_p]),
    "cw_release": (c_int32, [c_void_p, c_int32]),
    "cw_exec_duration_ns": (c_int32, [c_void_p, c_int32, POINTER(c_uint64)]),
    "cw_profile_measure": (c_int32, [c_void_p, c_int32, c_int32, c_int32, c_uint32, POINTER(cw_profile), c_void_p]),
    "cw_profile_get": (c_int32, [c_void_p, c_int32, c_int32, POINTER(cw_profile)]),
    "cw_plan_num_launches": (c_int32, [c_void_p, c_int32, c_int32]),
    "cw_plan_launch_info": (c_int32, [c_void_p, c_int32, c_int32, c_int32, POINTER(cw_launch_info)]),
    "cw_exec_timed_launches": (c_int32, [c_void_p, c_int32, c_int32, c_int32, c_int32, c_void_p, c_void_p]),
    "cw_debug_read_op": (c_int32, [c_void_p, c_int32, c_int32, c_int32, c_void_p, c_size_t]),
    "cw_set_debug_keep": (c_int32, [c_void_p, c_int32]),
    "cw_set_plan_override": (c_int32, [c_void_p, c_int32, c_int32]),
    "cw_set_plan_table": (c_int32, [c_void_p, c_void_p, c_int32]),
    "cw_set_fusion": (c_int32, [c_void_p, c_int32]),
    "cw_set_pair_launches": (c_int32, [c_void_p, c_int32]),
    "cw_set_panels": (c_int32, [c_void_p, c_int32]),
    "cw_set_fusion_third": (c_int32, [c_void_p, c_int32]),
    "cw_set_fusion_pool": (c_int32, [c_void_p, c_int32]),
    "cw_set_fusion_dw": (c_int32, [c_void_p, c_int32]),
    "cw_set_fc_softmax": (c_int32, [c_void_p, c_int32]),
    "cw_set_winograd": (c_int32, [c_void_p, c_int32]),
    "cw_set_resident": (c_int32, [c_void_p, c_int32]),
    "cw_set_use_graphs": (c_int32, [c_void_p, c_int32]),
    "cw_strerror": (c_char_p, [c_int32]),
    "cw_last_error": (c_char_p, [c_void_p]),
}

_lib = None


def lib():
    """The loaded library.  Builds it only if no built library exists; fails
    loudly if it cannot be had (there is no other implementation to fall to)."""
    global _lib
    if _lib is None:
        # PyTorch ships its own HIP runtime under the same soname.  Importing it first makes the
        # dynamic loader hand that one copy to this library too; loaded the other way round the
        # process would hold two HIP runtimes, and the second one fails to initialise.
        import torch  # noqa: F401
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        l = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


class CwError(RuntimeError):
    def __init__(self, status, detail=""):
        self.status = status
        name = lib().cw_strerror(status).decode()
        super().__init__("%s (%d)%s" % (name, status, (": " + detail) if detail else ""))


def _ptr(x):
    """Host address of a numpy array / torch CPU tensor / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return c_void_p(x)
    if isinstance(x, np.ndarray):
        assert x.flags["C_CONTIGUOUS"]
        return c_void_p(x.ctypes.data)
    if hasattr(x, "data_ptr"):
        assert x.is_contiguous()
        return c_void_p(x.data_ptr())
    raise TypeError(type(x))


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return c_void_p(s)
    return c_void_p(s.cuda_stream)  # torch.cuda.Stream


class Context:
    """One worker-GPU.  Methods carry the C names without the ``cw_`` prefix and
    raise :class:`CwError` on a negative status."""

    def __init__(self, device=0, workspace_bytes=512 << 20, io_bytes=512 << 20,
                 weight_pool_bytes=1 << 30, load_staging_bytes=256 << 20, weight_page_bytes=0):
        self._h = c_void_p()
        cfg = cw_config(device, workspace_bytes, io_bytes, weight_pool_bytes, load_staging_bytes, weight_page_bytes)
        st = lib().cw_create(byref(self._h), byref(cfg))
        if st != CW_OK:
            self._h = c_void_p()
            raise CwError(st, "cw_create: " + lib().cw_last_error(None).decode())

    def _check(self, st):
        if st < 0:
            raise CwError(st, lib().cw_last_error(self._h).decode())
        return st

    def destroy(self):
        if self._h:
            lib().cw_destroy(self._h)
            self._h = c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # -- models
    def model_define(self, ops, in_c, in_h, in_w, batch_sizes=(1, 2, 4, 8, 16), dtype="fp16"):
        arr = (cw_op * len(ops))(*[cw_op(*[int(v) for v in o]) for o in ops])
        bs = (c_int32 * len(batch_sizes))(*batch_sizes)
        mid = c_int32(-1)
        self._check(lib().cw_model_define(self._h, arr, len(ops), in_c, in_h, in_w, bs,
                                          len(batch_sizes), DTYPES[dtype], byref(mid)))
        return mid.value

    def model_define_resnet(self, depth, in_h, in_w, dtype="fp16"):
        mid = c_int32(-1)
        self._check(lib().cw_model_define_resnet(self._h, depth, in_h, in_w, DTYPES[dtype], byref(mid)))
        return mid.value

    def model_get_ops(self, model_id):
        n = c_int32(0)
        self._check(lib().cw_model_get_ops(self._h, model_id, None, 0, byref(n)))
        arr = (cw_op * n.value)()
        self._check(lib().cw_model_get_ops(self._h, model_id, arr, n.value, byref(n)))
        return [tuple(getattr(o, f) for f, _ in cw_op._fields_) for o in arr]

    def model_weight_bytes(self, model_id):
        return lib().cw_model_weight_bytes(self._h, model_id)

    def model_workspace_bytes(self, model_id, batch):
        return lib().cw_model_workspace_bytes(self._h, model_id, batch)

    # -- LOAD / UNLOAD
    def load_weights(self, model_id, host_blob, stream=None):
        nbytes = host_blob.nbytes if isinstance(host_blob, np.ndarray) else host_blob.numel() * host_blob.element_size()
        self._check(lib().cw_load_weights(self._h, model_id, _ptr(host_blob), nbytes, _stream(stream)))

    def load_weights_begin(self, model_id, host_blob, stream=None):
        """First step of a LOAD in steps; returns the handle the other three steps take."""
        nbytes = host_blob.nbytes if isinstance(host_blob, np.ndarray) else host_blob.numel() * host_blob.element_size()
        pending = c_void_p()
        self._check(lib().cw_load_weights_begin(self._h, model_id, _ptr(host_blob), nbytes, _stream(stream), ctypes.byref(pending)))
        return pending

    def load_weights_record(self, pending):
        self._check(lib().cw_load_weights_record(self._h, pending))

    def load_weights_end(self, pending):
        self._check(lib().cw_load_weights_end(self._h, pending))

    def load_weights_release(self, pending):
        lib().cw_load_weights_release(pending)

    def unload_weights(self, model_id):
        self._check(lib().cw_unload_weights(self._h, model_id))

    def weight_pool_free(self):
        return lib().cw_weight_pool_free(self._h)

    def weight_pages_free(self):
        return self._check(lib().cw_weight_pages_free(self._h))

    def model_weight_pages(self, model_id):
        return self._check(lib().cw_model_weight_pages(self._h, model_id))

    # -- INFER
    def input(self, model_id, batch, host_nchw, stream=None):
        slot = c_int32(-1)
        self._check(lib().cw_input(self._h, model_id, batch, _ptr(host_nchw), byref(slot), _stream(stream)))
        return slot.value

    def exec(self, model_id, batch, slot, stream=None):
        self._check(lib().cw_exec(self._h, model_id, batch, slot, _stream(stream)))

    def exec_static(self, model_id, batch, dev_input, dev_logits, dev_probs, stream=None):
        """dev_*: device tensors (anything with data_ptr()) or raw device addresses."""
        self._check(lib().cw_exec_static(self._h, model_id, batch, _ptr(dev_input), _ptr(dev_logits), _ptr(dev_probs),
                                         _stream(stream)))

    @staticmethod
    def exec_static_capacity():
        return lib().cw_exec_static_capacity()

    def output(self, slot, host_probs, host_logits=None, stream=None):
        self._check(lib().cw_output(self._h, slot, _ptr(host_probs), _ptr(host_logits), _stream(stream)))

    def release(self, slot):
        self._check(lib().cw_release(self._h, slot))

    def exec_duration_ns(self, slot):
        ns = c_uint64(0)
        self._check(lib().cw_exec_duration_ns(self._h, slot, byref(ns)))
        return ns.value

    # -- profile
    def profile_measure(self, model_id, batch, repeats, want_samples=False, slot=-1):
        prof = cw_profile()
        samples = np.empty(repeats, np.float32) if want_samples else None
        self._check(lib().cw_profile_measure(self._h, model_id, batch, slot, repeats, byref(prof), _ptr(samples)))
        d = {f: getattr(prof, f) for f, _ in cw_profile._fields_}
        return (d, samples) if want_samples else d

    def profile_get(self, model_id, batch):
        prof = cw_profile()
        self._check(lib().cw_profile_get(self._h, model_id, batch, byref(prof)))
        return {f: getattr(prof, f) for f, _ in cw_profile._fields_}

    # -- introspection
    def plan_num_launches(self, model_id, batch):
        return self._check(lib().cw_plan_num_launches(self._h, model_id, batch))

    def plan_launch_info(self, model_id, batch, index):
        info = cw_launch_info()
        self._check(lib().cw_plan_launch_info(self._h, model_id, batch, index, byref(info)))
        d = {f: getattr(info, f) for f, _ in cw_launch_info._fields_}
        d["name"] = d["name"].decode()
        return d

    def plan(self, model_id, batch):
        return [self.plan_launch_info(model_id, batch, i) for i in range(self.plan_num_launches(model_id, batch))]

    def exec_timed_launches(self, model_id, batch, slot, stream=None, inner=1):
        us = np.empty(self.plan_num_launches(model_id, batch), np.float32)
        self._check(lib().cw_exec_timed_launches(self._h, model_id, batch, slot, inner, _ptr(us), _stream(stream)))
        return us

    def debug_read_op(self, model_id, batch, op_index, shape):
        out = np.empty(shape, np.float32)
        self._check(lib().cw_debug_read_op(self._h, model_id, batch, op_index, _ptr(out), out.size))
        return out

    def set_debug_keep(self, keep):
        self._check(lib().cw_set_debug_keep(self._h, int(keep)))

    def set_use_graphs(self, on):
        self._check(lib().cw_set_use_graphs(self._h, int(on)))

    def set_plan_override(self, conv_tile=-1, split_k=0):
        if isinstance(conv_tile, str):
            conv_tile = CONV_TILES[conv_tile]
        self._check(lib().cw_set_plan_override(self._h, conv_tile, split_k))

    def set_pair_launches(self, on):
        self._check(lib().cw_set_pair_launches(self._h, int(on)))

    def set_fc_softmax(self, on):
        self._check(lib().cw_set_fc_softmax(self._h, int(on)))

    def set_fusion_third(self, on):
        self._check(lib().cw_set_fusion_third(self._h, int(on)))

    def set_fusion_pool(self, on):
        self._check(lib().cw_set_fusion_pool(self._h, int(on)))

    def set_fusion_dw(self, on):
        self._check(lib().cw_set_fusion_dw(self._h, int(on)))

    def set_panels(self, on):
        self._check(lib().cw_set_panels(self._h, int(on)))

    def set_resident(self, on):
        self._check(lib().cw_set_resident(self._h, int(on)))

    def set_winograd(self, on):
        self._check(lib().cw_set_winograd(self._h, int(on)))

    def set_fusion(self, on):
        self._check(lib().cw_set_fusion(self._h, int(on)))

    def set_plan_table(self, rows):
        """rows: iterable of (M, N, K, kh, stride, conv_tile, split_k); empty removes the table."""
        arr = np.ascontiguousarray(np.array([[CONV_TILES[v] if isinstance(v, str) else v for v in r] for r in rows],
                                            dtype=np.int32).reshape(-1, 7))
        self._check(lib().cw_set_plan_table(self._h, _ptr(arr) if len(arr) else None, len(arr)))


__all__ = [n for n in dir() if n.startswith("CW_") or n.startswith("cw_")] + [
    "Context", "CwError", "lib", "LIB_PATH", "SIGNATURES", "DTYPES", "CONV_TILES"]


class Executors:
    """The worker's executors over one Context (C names without the ``cw_worker_`` prefix).  Host
    buffers of submitted actions are kept alive here until their results have been fetched."""

    def __init__(self, ctx, cores=None):
        self._ctx = ctx
        self._h = c_void_p()
        arr = (c_int32 * 5)(*cores) if cores is not None else None
        st = lib().cw_worker_create(ctx._h, arr, byref(self._h))
        if st < 0:
            raise CwError(st, "cw_worker_create")
        self._keep = {}

    @staticmethod
    def now_ns():
        return lib().cw_worker_now_ns()

    def submit(self, action_id, type, model_id, earliest_ns, latest_ns, batch=0, host_in=None, host_probs=None, host_logits=None):
        nbytes = 0
        if host_in is not None:
            nbytes = host_in.nbytes if isinstance(host_in, np.ndarray) else host_in.numel() * host_in.element_size()
        a = cw_action(action_id, type, model_id, batch, earliest_ns, latest_ns, _ptr(host_in), nbytes, _ptr(host_probs), _ptr(host_logits))
        self._keep[action_id] = (host_in, host_probs, host_logits)
        st = lib().cw_worker_submit(self._h, byref(a))
        if st < 0:
            self._keep.pop(action_id, None)
            raise CwError(st, "cw_worker_submit")

    def next_result(self, timeout_s=5.0):
        """dict of the next finished action, or None after the time-out."""
        r = cw_result()
        st = lib().cw_worker_next_result(self._h, byref(r), int(timeout_s * 1e9))
        if st == CW_ERR_TIMEOUT:
            return None
        if st < 0:
            raise CwError(st, "cw_worker_next_result")
        self._keep.pop(r.id, None)
        return {f: getattr(r, f) for f, _ in cw_result._fields_}

    def profile(self, type, model_id, batch=0):
        n, mean, mx = c_uint32(0), c_uint64(0), c_uint64(0)
        st = lib().cw_worker_profile(self._h, type, model_id, batch, byref(n), byref(mean), byref(mx))
        if st < 0:
            raise CwError(st, "cw_worker_profile")
        return {"n": n.value, "mean_ns": mean.value, "max_ns": mx.value}

    def destroy(self):
        if self._h:
            lib().cw_worker_destroy(self._h)
            self._h = c_void_p()
            self._keep.clear()
