"""ctypes binding with the same names as include/pp_deep_reuse.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
from typing import Optional

import numpy as np

from .pp_conv import PP_OK, PP_FLAG_HOST_ONLY, PP_FLAG_RELU, PPError, lib as _conv_lib


class _Desc(C.Structure):
    _fields_ = [("k", C.c_int32), ("m", C.c_int32), ("seg_len", C.c_int32), ("hash_bits", C.c_int32), ("n_max", C.c_int32),
                ("weights", C.c_void_p), ("bias", C.c_void_p), ("hyperplanes", C.c_void_p), ("flags", C.c_uint32)]


_ready = False


def lib() -> C.CDLL:
    global _ready
    L = _conv_lib()
    if not _ready:
        vp = C.c_void_p
        L.pp_reuse_plan.argtypes = [C.POINTER(_Desc), C.POINTER(vp)]
        L.pp_reuse_plan.restype = C.c_int
        L.pp_reuse_run.argtypes = [vp, vp, vp, C.c_int32, vp]
        L.pp_reuse_run.restype = C.c_int
        L.pp_reuse_read_clusters.argtypes = [vp, C.c_int32, vp, vp]
        L.pp_reuse_read_clusters.restype = C.c_int
        L.pp_reuse_destroy.argtypes = [vp]
        L.pp_reuse_destroy.restype = C.c_int
        _ready = True
    return L


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def pp_reuse_plan(k, m, seg_len, hash_bits, n_max, weights, bias, hyperplanes, flags=0):
    """Returns (status, handle)."""
    w = None if weights is None else np.ascontiguousarray(weights, dtype=np.float32)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    hp = None if hyperplanes is None else np.ascontiguousarray(hyperplanes, dtype=np.float32)
    d = _Desc(k, m, seg_len, hash_bits, n_max, _ptr(w), _ptr(b), _ptr(hp), flags)
    h = C.c_void_p()
    st = lib().pp_reuse_plan(C.byref(d), C.byref(h))
    return st, (h if st == PP_OK else None)


def pp_reuse_run(plan, x_dev: int, y_dev: int, n: int, hip_stream: int = 0) -> int:
    return lib().pp_reuse_run(plan, C.c_void_p(x_dev), C.c_void_p(y_dev), n, C.c_void_p(hip_stream))


def pp_reuse_read_clusters(plan, n: int, segments: int, hash_bits: int):
    """Returns (status, signatures [n, segments] uint16, representatives [segments, 2**hash_bits] int32)."""
    sig = np.empty((n, segments), dtype=np.uint16)
    rep = np.empty((segments, 1 << hash_bits), dtype=np.int32)
    st = lib().pp_reuse_read_clusters(plan, n, _ptr(sig), _ptr(rep))
    return st, sig, rep


def pp_reuse_destroy(plan) -> int:
    return lib().pp_reuse_destroy(plan)


class ReusePlan:
    """Owns one plan handle; run() takes torch tensors only to read their device pointers."""

    def __init__(self, handle, k, m, seg_len, hash_bits, n_max):
        self.handle, self.k, self.m, self.seg_len, self.hash_bits, self.n_max = handle, k, m, seg_len, hash_bits, n_max

    def run(self, x, y=None, stream: Optional[int] = None):
        import torch
        assert x.is_cuda and x.is_contiguous() and x.dtype == torch.float32 and x.dim() == 2 and x.shape[1] == self.k
        n = x.shape[0]
        if y is None:
            y = torch.empty((n, self.m), dtype=torch.float32, device=x.device)
        assert y.is_cuda and y.is_contiguous() and y.dtype == torch.float32 and tuple(y.shape) == (n, self.m)
        if stream is None:
            stream = torch.cuda.current_stream(x.device).cuda_stream
        st = pp_reuse_run(self.handle, x.data_ptr(), y.data_ptr(), n, stream)
        if st != PP_OK:
            raise PPError(st, "pp_reuse_run")
        return y

    def clusters(self, n):
        st, sig, rep = pp_reuse_read_clusters(self.handle, n, self.k // self.seg_len, self.hash_bits)
        if st != PP_OK:
            raise PPError(st, "pp_reuse_read_clusters")
        return sig, rep

    def close(self):
        if self.handle is not None:
            pp_reuse_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def reuse_plan_from_layer(layer, host_only=False, n_max=None) -> ReusePlan:
    """Plan for a deep-reuse layer description object (fields as in synth.ReuseLayer)."""
    flags = (PP_FLAG_RELU if layer.relu else 0) | (PP_FLAG_HOST_ONLY if host_only else 0)
    n_max = layer.n if n_max is None else n_max
    st, h = pp_reuse_plan(layer.k, layer.m, layer.seg_len, layer.hash_bits, n_max, layer.weights, layer.bias, layer.hyperplanes, flags)
    if st != PP_OK:
        raise PPError(st, "pp_reuse_plan")
    return ReusePlan(h, layer.k, layer.m, layer.seg_len, layer.hash_bits, n_max)
