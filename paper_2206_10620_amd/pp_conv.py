"""ctypes binding with the same names as include/pp_conv.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

PP_OK, PP_ERR_NULL, PP_ERR_SHAPE, PP_ERR_PATTERN, PP_ERR_UNSUPPORTED, PP_ERR_ALLOC, PP_ERR_DEVICE, PP_ERR_ALIGN, PP_ERR_SCRATCH = range(9)
PP_F32, PP_F16 = 0, 1
PP_FLAG_RELU, PP_FLAG_DENSE, PP_FLAG_HOST_ONLY, PP_FLAG_POOL2 = 1, 2, 4, 8

# Bumped whenever the device code of the tiled kernel changes (measurements that are tied to a
# kernel build, such as hardware-counter readings, are keyed by it).
KERNEL_REVISION = "lib-2026-11-28-i"

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpp_conv.so")


class PPError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {pp_status_string(status)} (status {status})")


class Tuning(C.Structure):
    _fields_ = [("variant", C.c_int32), ("filters_per_wave", C.c_int32), ("rows_per_lane", C.c_int32),
                ("lanes_x", C.c_int32), ("waves_f", C.c_int32), ("split_c", C.c_int32), ("chunk_c", C.c_int32),
                ("staging", C.c_int32), ("split_wg", C.c_int32), ("balance", C.c_int32),
                ("tile_rows", C.c_int32), ("tile_cols", C.c_int32), ("tiles_per_wave", C.c_int32),
                ("wg_waves", C.c_int32), ("autotune", C.c_int32), ("mfma_kind", C.c_int32), ("split_k", C.c_int32)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class _Desc(C.Structure):
    _fields_ = [("c_in", C.c_int32), ("c_out", C.c_int32), ("h", C.c_int32), ("w", C.c_int32),
                ("n_hint", C.c_int32), ("num_patterns", C.c_int32),
                ("pattern_masks", C.c_void_p), ("pattern_id", C.c_void_p), ("conn_mask", C.c_void_p),
                ("weights", C.c_void_p), ("bias", C.c_void_p),
                ("flags", C.c_uint32), ("dtype", C.c_int32), ("tuning", C.POINTER(Tuning)),
                ("kernel_size", C.c_int32), ("stride", C.c_int32), ("taps_per_kernel", C.c_int32),
                ("pattern_masks64", C.c_void_p)]


class _Info(C.Structure):
    _fields_ = [("c_out", C.c_int32), ("c_in", C.c_int32), ("num_patterns", C.c_int32), ("taps", C.c_int32),
                ("out_h", C.c_int32), ("out_w", C.c_int32), ("k_kept", C.c_int64),
                ("perm", C.POINTER(C.c_int32)), ("kcount", C.POINTER(C.c_int32)), ("pat_off", C.POINTER(C.c_int32)),
                ("kidx", C.POINTER(C.c_int32)), ("kpat", C.POINTER(C.c_uint8)), ("wpacked", C.POINTER(C.c_float)),
                ("chosen", Tuning)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def lib() -> C.CDLL:
    """The loaded HIP library.  Raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2206_10620_amd.build` "
                              "(hipcc, gfx950); this package has no CPU fallback")
        L = C.CDLL(_LIB_PATH)
        vp = C.c_void_p
        L.pp_conv_plan.argtypes = [C.POINTER(_Desc), C.POINTER(vp)]
        L.pp_conv_plan.restype = C.c_int
        L.pp_conv_run.argtypes = [vp, vp, vp, C.c_int32, vp]
        L.pp_conv_run.restype = C.c_int
        L.pp_conv_run_static.argtypes = [vp, vp, vp, C.c_int32, vp]
        L.pp_conv_run_static.restype = C.c_int
        L.pp_conv_destroy.argtypes = [vp]
        L.pp_conv_destroy.restype = C.c_int
        L.pp_conv_plan_query.argtypes = [vp, C.POINTER(_Info)]
        L.pp_conv_plan_query.restype = C.c_int
        L.pp_conv_plan_unpack.argtypes = [vp, vp, vp, vp]
        L.pp_conv_plan_unpack.restype = C.c_int
        L.pp_maxpool2x2_run.argtypes = [vp, vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp]
        L.pp_maxpool2x2_run.restype = C.c_int
        L.pp_status_string.argtypes = [C.c_int]
        L.pp_status_string.restype = C.c_char_p
        _lib = L
    return _lib


def pp_status_string(status: int) -> str:
    return lib().pp_status_string(int(status)).decode()


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def pp_conv_plan(c_in, c_out, h, w, pattern_masks, pattern_id, conn_mask, weights, bias=None, flags=0,
                 dtype=PP_F32, n_hint=1, tuning: Optional[Tuning] = None, kernel_size=0, stride=0, taps_per_kernel=0):
    """Returns (status, plan handle or None).  Array arguments are numpy arrays (or None where the
    header allows NULL); they are converted to the C element types without any other processing."""
    keep = []

    def arr(a, dt):
        if a is None:
            return None
        b = np.ascontiguousarray(a, dtype=dt)
        keep.append(b)
        return b

    d = _Desc()
    d.c_in, d.c_out, d.h, d.w, d.n_hint = int(c_in), int(c_out), int(h), int(w), int(n_hint)
    wide = int(kernel_size) > 3                      # 25- and 49-bit masks travel as 64-bit words
    masks = arr(pattern_masks, np.uint64 if wide else np.uint16)
    d.num_patterns = 0 if masks is None else int(masks.size)
    d.pattern_masks = None if wide else _ptr(masks)
    d.pattern_masks64 = _ptr(masks) if wide else None
    d.kernel_size, d.stride, d.taps_per_kernel = int(kernel_size), int(stride), int(taps_per_kernel)
    d.pattern_id = _ptr(arr(pattern_id, np.int32))
    d.conn_mask = _ptr(arr(conn_mask, np.uint8))
    d.weights = _ptr(arr(weights, np.float32))
    d.bias = _ptr(arr(bias, np.float32))
    d.flags, d.dtype = int(flags), int(dtype)
    d.tuning = C.pointer(tuning) if tuning is not None else None
    out = C.c_void_p()
    st = lib().pp_conv_plan(C.byref(d), C.byref(out))
    return st, (out if st == PP_OK else None)


def pp_conv_run(plan, x_dev: int, y_dev: int, n: int, hip_stream: int = 0) -> int:
    return lib().pp_conv_run(plan, C.c_void_p(x_dev), C.c_void_p(y_dev), int(n), C.c_void_p(hip_stream))


def pp_conv_run_static(plan, x_dev: int, y_dev: int, n: int, hip_stream: int = 0) -> int:
    return lib().pp_conv_run_static(plan, C.c_void_p(x_dev), C.c_void_p(y_dev), int(n), C.c_void_p(hip_stream))


def pp_conv_destroy(plan) -> int:
    return lib().pp_conv_destroy(plan)


def pp_conv_plan_query(plan):
    """Returns (status, dict of numpy copies of the canonical plan arrays)."""
    info = _Info()
    st = lib().pp_conv_plan_query(plan, C.byref(info))
    if st != PP_OK:
        return st, None
    P, co, kk, taps = info.num_patterns, info.c_out, info.k_kept, info.taps

    def grab(ptr, count, dt):
        if count == 0:
            return np.zeros(0, dtype=dt)
        return np.ctypeslib.as_array(ptr, shape=(count,)).astype(dt, copy=True)

    return st, dict(c_out=co, c_in=info.c_in, num_patterns=P, taps=taps, k_kept=kk, out_h=info.out_h, out_w=info.out_w,
                    perm=grab(info.perm, co, np.int32), kcount=grab(info.kcount, co, np.int32),
                    pat_off=grab(info.pat_off, co * (P + 1), np.int32).reshape(co, P + 1),
                    kidx=grab(info.kidx, kk, np.int32), kpat=grab(info.kpat, kk, np.uint8),
                    wpacked=grab(info.wpacked, kk * taps, np.float32).reshape(kk, taps),
                    chosen=info.chosen.as_dict())


def pp_conv_plan_unpack(plan, k_kept: int):
    kidx = np.empty(k_kept, np.int32)
    kpat = np.empty(k_kept, np.uint8)
    w = np.empty((k_kept, 4), np.float32)
    st = lib().pp_conv_plan_unpack(plan, _ptr(kidx), _ptr(kpat), _ptr(w))
    return st, kidx, kpat, w


def pp_maxpool2x2_run(x_dev: int, y_dev: int, n, c, h, w, dtype, hip_stream: int = 0) -> int:
    return lib().pp_maxpool2x2_run(C.c_void_p(x_dev), C.c_void_p(y_dev), int(n), int(c), int(h), int(w), int(dtype),
                                   C.c_void_p(hip_stream))


class Plan:
    """Owns one plan handle; run() takes torch tensors only to read their device pointers."""

    def __init__(self, handle, c_in, c_out, h, w, dtype):
        self.handle, self.c_in, self.c_out, self.h, self.w, self.dtype = handle, c_in, c_out, h, w, dtype
        info = self.query()
        self.out_h, self.out_w = info["out_h"], info["out_w"]

    def query(self):
        st, info = pp_conv_plan_query(self.handle)
        if st != PP_OK:
            raise PPError(st, "pp_conv_plan_query")
        return info

    def run(self, x, y=None, stream: Optional[int] = None, static: bool = False):
        """static=True goes through pp_conv_run_static (y must then be given: that entry point is for
        callers that allocate nothing)."""
        import torch
        tdt = torch.float16 if self.dtype == PP_F16 else torch.float32
        assert x.is_cuda and x.is_contiguous() and x.dtype == tdt and tuple(x.shape[1:]) == (self.c_in, self.h, self.w)
        n = x.shape[0]
        if y is None:
            y = torch.empty((n, self.c_out, self.out_h, self.out_w), dtype=tdt, device=x.device)
        assert y.is_cuda and y.is_contiguous() and y.dtype == tdt and tuple(y.shape) == (n, self.c_out, self.out_h, self.out_w)
        if stream is None:
            stream = torch.cuda.current_stream(x.device).cuda_stream
        st = (pp_conv_run_static if static else pp_conv_run)(self.handle, x.data_ptr(), y.data_ptr(), n, stream)
        if st != PP_OK:
            raise PPError(st, "pp_conv_run_static" if static else "pp_conv_run")
        return y

    def close(self):
        if self.handle is not None:
            pp_conv_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def plan_from_layer(layer, host_only=False, tuning: Optional[Tuning] = None, n_hint: Optional[int] = None) -> Plan:
    """Plan for a layer description object (fields as in synth.Layer)."""
    flags = (PP_FLAG_RELU if layer.relu else 0) | (PP_FLAG_DENSE if layer.dense else 0) | \
            (PP_FLAG_HOST_ONLY if host_only else 0) | (PP_FLAG_POOL2 if getattr(layer, "pool", False) else 0)
    dtype = PP_F16 if layer.dtype == "f16" else PP_F32
    st, h = pp_conv_plan(layer.c_in, layer.c_out, layer.h, layer.w, layer.pattern_masks, layer.pattern_id,
                         layer.conn_mask, layer.weights, layer.bias, flags, dtype,
                         layer.n if n_hint is None else n_hint, tuning, getattr(layer, "ksize", 3),
                         getattr(layer, "stride", 1), 0 if layer.dense else layer.taps)
    if st != PP_OK:
        raise PPError(st, "pp_conv_plan")
    return Plan(h, layer.c_in, layer.c_out, layer.h, layer.w, dtype)
