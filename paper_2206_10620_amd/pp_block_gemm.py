"""ctypes binding with the same names as include/pp_block_gemm.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
from typing import Optional

import numpy as np

from .pp_conv import PP_OK, PP_F16, PP_F32, PP_FLAG_HOST_ONLY, PP_FLAG_RELU, PPError, lib as _conv_lib


# Bumped whenever the device code of the matrix-core kernel changes (hardware-counter readings are keyed by it).
BLOCK_KERNEL_REVISION = "k4-2026-11-28-b"


class _Desc(C.Structure):
    _fields_ = [("m", C.c_int32), ("k", C.c_int32), ("block_m", C.c_int32), ("block_k", C.c_int32),
                ("row_keep", C.c_void_p), ("col_keep", C.c_void_p), ("weights", C.c_void_p), ("bias", C.c_void_p),
                ("flags", C.c_uint32), ("dtype", C.c_int32), ("variant", C.c_int32)]


class _Info(C.Structure):
    _fields_ = [("m", C.c_int32), ("k", C.c_int32), ("block_m", C.c_int32), ("block_k", C.c_int32),
                ("variant", C.c_int32), ("row_tile", C.c_int32), ("row_tiles", C.c_int32),
                ("kept_weights", C.c_int64), ("executed_weights", C.c_int64),
                ("tile_off", C.POINTER(C.c_int32)), ("tile_cols", C.POINTER(C.c_int32)), ("tile_len", C.POINTER(C.c_int32))]


_ready = False


def lib() -> C.CDLL:
    """The loaded HIP library (the same shared object as the convolution's; no fallback)."""
    global _ready
    L = _conv_lib()
    if not _ready:
        vp = C.c_void_p
        L.pp_block_gemm_plan.argtypes = [C.POINTER(_Desc), C.POINTER(vp)]
        L.pp_block_gemm_plan.restype = C.c_int
        L.pp_block_gemm_run.argtypes = [vp, vp, vp, C.c_int32, vp]
        L.pp_block_gemm_run.restype = C.c_int
        L.pp_block_gemm_destroy.argtypes = [vp]
        L.pp_block_gemm_destroy.restype = C.c_int
        L.pp_block_gemm_query.argtypes = [vp, C.POINTER(_Info)]
        L.pp_block_gemm_query.restype = C.c_int
        L.pp_block_gemm_unpack.argtypes = [vp, C.c_int32, vp]
        L.pp_block_gemm_unpack.restype = C.c_int
        _ready = True
    return L


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def pp_block_gemm_plan(m, k, block_m, block_k, row_keep, col_keep, weights, bias=None, flags=0, dtype=PP_F16, variant=0):
    """Returns (status, handle)."""
    rk = None if row_keep is None else np.ascontiguousarray(row_keep, dtype=np.uint8)
    ck = None if col_keep is None else np.ascontiguousarray(col_keep, dtype=np.uint8)
    w = None if weights is None else np.ascontiguousarray(weights, dtype=np.float32)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    d = _Desc(m, k, block_m, block_k, _ptr(rk), _ptr(ck), _ptr(w), _ptr(b), flags, dtype, variant)
    h = C.c_void_p()
    st = lib().pp_block_gemm_plan(C.byref(d), C.byref(h))
    return st, (h if st == PP_OK else None)


def pp_block_gemm_run(plan, x_dev: int, y_dev: int, n: int, hip_stream: int = 0) -> int:
    return lib().pp_block_gemm_run(plan, C.c_void_p(x_dev), C.c_void_p(y_dev), n, C.c_void_p(hip_stream))


def pp_block_gemm_destroy(plan) -> int:
    return lib().pp_block_gemm_destroy(plan)


def pp_block_gemm_query(plan):
    """Returns (status, dict) with the lists copied into numpy arrays."""
    info = _Info()
    st = lib().pp_block_gemm_query(plan, C.byref(info))
    if st != PP_OK:
        return st, None
    rt = info.row_tiles
    off = np.ctypeslib.as_array(info.tile_off, shape=(rt + 1,)).copy()
    total = int(off[-1])
    cols = np.ctypeslib.as_array(info.tile_cols, shape=(total,)).copy() if total else np.zeros(0, np.int32)
    length = np.ctypeslib.as_array(info.tile_len, shape=(rt,)).copy()
    return st, dict(m=info.m, k=info.k, block_m=info.block_m, block_k=info.block_k, variant=info.variant, row_tile=info.row_tile,
                    row_tiles=rt, kept_weights=info.kept_weights, executed_weights=info.executed_weights, tile_off=off,
                    tile_cols=cols, tile_len=length)


def pp_block_gemm_unpack(plan, tile: int, row_tile: int, k: int):
    out = np.empty((row_tile, k), dtype=np.float32)
    st = lib().pp_block_gemm_unpack(plan, tile, _ptr(out))
    return st, out


class BlockPlan:
    """Owns one plan handle; run() takes torch tensors only to read their device pointers."""

    def __init__(self, handle, m, k, dtype):
        self.handle, self.m, self.k, self.dtype = handle, m, k, dtype

    def query(self):
        st, info = pp_block_gemm_query(self.handle)
        if st != PP_OK:
            raise PPError(st, "pp_block_gemm_query")
        return info

    def run(self, x, y=None, stream: Optional[int] = None):
        import torch
        tdt = torch.float16 if self.dtype == PP_F16 else torch.float32
        assert x.is_cuda and x.is_contiguous() and x.dtype == tdt and x.dim() == 2 and x.shape[0] == self.k
        n = x.shape[1]
        if y is None:
            y = torch.empty((self.m, n), dtype=tdt, device=x.device)
        assert y.is_cuda and y.is_contiguous() and y.dtype == tdt and tuple(y.shape) == (self.m, n)
        if stream is None:
            stream = torch.cuda.current_stream(x.device).cuda_stream
        st = pp_block_gemm_run(self.handle, x.data_ptr(), y.data_ptr(), n, stream)
        if st != PP_OK:
            raise PPError(st, "pp_block_gemm_run")
        return y

    def close(self):
        if self.handle is not None:
            pp_block_gemm_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def block_plan_from_layer(layer, host_only=False, variant=0) -> BlockPlan:
    """Plan for a block-layer description object (fields as in synth.BlockLayer)."""
    flags = (PP_FLAG_RELU if layer.relu else 0) | (PP_FLAG_HOST_ONLY if host_only else 0)
    dtype = PP_F16 if layer.dtype == "f16" else PP_F32
    st, h = pp_block_gemm_plan(layer.m, layer.k, layer.bm, layer.bk, layer.row_keep, layer.col_keep, layer.weights, layer.bias,
                               flags, dtype, variant)
    if st != PP_OK:
        raise PPError(st, "pp_block_gemm_plan")
    return BlockPlan(h, layer.m, layer.k, dtype)
