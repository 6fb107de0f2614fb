"""ctypes wrapper around libpp_oracle.so (built from pp_oracle.cpp with g++)."""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pp_oracle.cpp")
_SRC_BLOCK = os.path.join(_HERE, "pp_block_oracle.cpp")
_SRC_REUSE = os.path.join(_HERE, "pp_reuse_oracle.cpp")
_SO = os.path.join(_HERE, "libpp_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the checker (host compiler only)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_BLOCK), os.path.getmtime(_SRC_REUSE))
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < newest:
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread", "-ffp-contract=off", "-o", _SO, _SRC, _SRC_BLOCK, _SRC_REUSE])
    return _SO


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_SO)
        vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
        L.oracle_expand_weights.argtypes = [i32, i32, i32, vp, vp, vp, vp, i32, vp]
        L.oracle_expand_weights.restype = i32
        L.oracle_conv.argtypes = [i32] * 5 + [vp, vp, vp, i32, vp, vp, vp, i32]
        L.oracle_conv.restype = None
        L.oracle_conv_at.argtypes = [i32] * 5 + [vp, vp, i32, i32, vp, i64, vp, vp, vp, vp, i32]
        L.oracle_conv_at.restype = None
        L.oracle_brute.argtypes = [i32] * 6 + [vp] * 6 + [i32, vp]
        L.oracle_brute.restype = None
        L.oracle_maxpool2.argtypes = [i32] * 4 + [vp, vp]
        L.oracle_maxpool2.restype = None
        L.oracle_round_f16.argtypes = [i64, vp, vp]
        L.oracle_round_f16.restype = None
        L.oracle_widen_f16.argtypes = [i64, vp, vp]
        L.oracle_widen_f16.restype = None
        L.oracle_plan_ref.argtypes = [i32, i32, i32] + [vp] * 8
        L.oracle_plan_ref.restype = i64
        L.oracle_expand_weights_k.argtypes = [i32] * 5 + [vp] * 5
        L.oracle_expand_weights_k.restype = i32
        L.oracle_conv_k.argtypes = [i32] * 7 + [vp, vp, vp, i32, vp, vp, vp, i32]
        L.oracle_conv_k.restype = None
        L.oracle_conv_k_at.argtypes = [i32] * 7 + [vp, vp, i32, i32, vp, i64, vp, vp, vp, vp, i32]
        L.oracle_conv_k_at.restype = None
        L.oracle_brute_k.argtypes = [i32] * 8 + [vp] * 6 + [i32, vp]
        L.oracle_brute_k.restype = None
        L.oracle_block_expand.argtypes = [i32] * 4 + [vp] * 4
        L.oracle_block_expand.restype = i32
        L.oracle_gemm.argtypes = [i32] * 3 + [vp] * 3 + [i32] + [vp] * 3 + [i32]
        L.oracle_gemm.restype = None
        L.oracle_gemm_at.argtypes = [i32] * 3 + [vp] * 3 + [i32, vp, i64] + [vp] * 3 + [i32]
        L.oracle_gemm_at.restype = None
        L.oracle_block_brute.argtypes = [i32] * 5 + [vp] * 5 + [i32, vp]
        L.oracle_block_brute.restype = None
        L.oracle_reuse_signatures.argtypes = [i32] * 4 + [vp] * 3
        L.oracle_reuse_signatures.restype = i32
        L.oracle_reuse_representatives.argtypes = [i32] * 3 + [vp] * 2
        L.oracle_reuse_representatives.restype = None
        L.oracle_reuse_apply.argtypes = [i32] * 5 + [vp] * 5 + [i32] + [vp] * 3
        L.oracle_reuse_apply.restype = None
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def default_threads() -> int:
    try:
        return max(1, len(os.sched_getaffinity(0)))
    except AttributeError:
        return os.cpu_count() or 1


def expand_weights(c_in, c_out, masks, pattern_id, conn, weights, taps=4) -> np.ndarray:
    """Masked dense weights Wd [c_out, c_in, 3, 3] (float64)."""
    masks = _c(masks, np.uint16)
    pid = _c(pattern_id, np.int32)
    cm = _c(conn, np.uint8)
    w = _c(weights, np.float64).reshape(-1)
    wd = np.empty((c_out, c_in, 3, 3), dtype=np.float64)
    rc = lib().oracle_expand_weights(c_in, c_out, len(masks), _p(masks), _p(pid), _p(cm), _p(w), taps, _p(wd))
    if rc != 0:
        raise ValueError(f"invalid pruned-layer description (code {rc})")
    return wd


def conv(x, wd, bias=None, relu=False, want_pre=False, want_scale=False, threads=None):
    """Full-tensor reference result.  Returns y, or (y, pre, scale) with the extras asked for."""
    x = _c(x, np.float64)
    wd = _c(wd, np.float64)
    n, c_in, h, w = x.shape
    c_out = wd.shape[0]
    assert wd.shape == (c_out, c_in, 3, 3)
    b = None if bias is None else _c(bias, np.float64)
    y = np.empty((n, c_out, h, w), dtype=np.float64)
    pre = np.empty_like(y) if want_pre else None
    sc = np.empty_like(y) if want_scale else None
    lib().oracle_conv(n, c_in, c_out, h, w, _p(x), _p(wd), _p(b), int(relu), _p(y), _p(pre), _p(sc),
                      threads or default_threads())
    if want_pre or want_scale:
        return y, pre, sc
    return y


def conv_at(x, wd, pts, bias=None, relu=False, threads=None):
    """Reference result at sampled outputs.  x is float32 or float16 [n,c_in,h,w];
    pts int32 [npts, 4] of (n, co, oy, ox).  Returns (y, pre, scale)."""
    assert x.dtype in (np.float32, np.float16) and x.flags.c_contiguous
    wd = _c(wd, np.float64)
    n, c_in, h, w = x.shape
    c_out = wd.shape[0]
    pts = _c(pts, np.int32)
    npts = pts.shape[0]
    b = None if bias is None else _c(bias, np.float64)
    y = np.empty(npts, dtype=np.float64)
    pre = np.empty(npts, dtype=np.float64)
    sc = np.empty(npts, dtype=np.float64)
    lib().oracle_conv_at(n, c_in, c_out, h, w, _p(wd), _p(b), int(relu), int(x.dtype == np.float16), _p(x), npts,
                         _p(pts), _p(y), _p(pre), _p(sc), threads or default_threads())
    return y, pre, sc


def brute(x, masks, pattern_id, conn, weights, c_out, bias=None, relu=False):
    x = _c(x, np.float64)
    n, c_in, h, w = x.shape
    masks = _c(masks, np.uint16)
    pid = _c(pattern_id, np.int32)
    cm = _c(conn, np.uint8)
    wt = _c(weights, np.float64).reshape(-1)
    b = None if bias is None else _c(bias, np.float64)
    y = np.empty((n, c_out, h, w), dtype=np.float64)
    lib().oracle_brute(n, c_in, c_out, h, w, len(masks), _p(masks), _p(pid), _p(cm), _p(wt), _p(x), _p(b),
                       int(relu), _p(y))
    return y


def maxpool2(x):
    x = _c(x, np.float64)
    n, c, h, w = x.shape
    y = np.empty((n, c, h // 2, w // 2), dtype=np.float64)
    lib().oracle_maxpool2(n, c, h, w, _p(x), _p(y))
    return y


def round_f16(v) -> np.ndarray:
    """Round float64 values to IEEE binary16 (nearest even); returns uint16 bit patterns."""
    v = _c(v, np.float64)
    out = np.empty(v.shape, dtype=np.uint16)
    lib().oracle_round_f16(v.size, _p(v), _p(out))
    return out


def widen_f16(bits) -> np.ndarray:
    bits = _c(bits, np.uint16)
    out = np.empty(bits.shape, dtype=np.float64)
    lib().oracle_widen_f16(bits.size, _p(bits), _p(out))
    return out


def plan_ref(c_in, c_out, num_patterns, pattern_id, conn):
    """Reference filter-kernel ordering; dict of canonical arrays."""
    pid = _c(pattern_id, np.int32)
    cm = _c(conn, np.uint8)
    kk = int(np.count_nonzero(cm))
    perm = np.empty(c_out, np.int32)
    kcount = np.empty(c_out, np.int32)
    pat_off = np.empty(c_out * (num_patterns + 1), np.int32)
    kidx = np.empty(kk, np.int32)
    kpat = np.empty(kk, np.uint8)
    wsel = np.empty(kk, np.int64)
    got = lib().oracle_plan_ref(c_in, c_out, num_patterns, _p(pid), _p(cm), _p(perm), _p(kcount), _p(pat_off),
                                _p(kidx), _p(kpat), _p(wsel))
    assert got == kk
    return dict(perm=perm, kcount=kcount, pat_off=pat_off.reshape(c_out, num_patterns + 1), kidx=kidx, kpat=kpat,
                wsel=wsel, k_kept=kk)


# -- other kernel sizes and strides -------------------------------------------------------

def out_size(size: int, stride: int) -> int:
    return (size - 1) // stride + 1


def expand_weights_k(c_in, c_out, ksize, masks, pattern_id, conn, weights, taps) -> np.ndarray:
    """Masked dense weights Wd [c_out, c_in, K, K] (float64) from (K*K)-bit masks."""
    masks = _c(masks, np.uint64)
    pid = _c(pattern_id, np.int32)
    cm = _c(conn, np.uint8)
    w = _c(weights, np.float64).reshape(-1)
    wd = np.empty((c_out, c_in, ksize, ksize), dtype=np.float64)
    rc = lib().oracle_expand_weights_k(c_in, c_out, ksize, taps, len(masks), _p(masks), _p(pid), _p(cm), _p(w), _p(wd))
    if rc != 0:
        raise ValueError(f"invalid pruned-layer description (code {rc})")
    return wd


def conv_k(x, wd, stride=1, bias=None, relu=False, want_pre=False, want_scale=False, threads=None):
    """Full-tensor reference result for K x K kernels (K = wd.shape[-1]), padding (K-1)/2, the given stride."""
    x = _c(x, np.float64)
    wd = _c(wd, np.float64)
    n, c_in, h, w = x.shape
    c_out, _, ksize, _ = wd.shape
    assert wd.shape == (c_out, c_in, ksize, ksize)
    b = None if bias is None else _c(bias, np.float64)
    y = np.empty((n, c_out, out_size(h, stride), out_size(w, stride)), dtype=np.float64)
    pre = np.empty_like(y) if want_pre else None
    sc = np.empty_like(y) if want_scale else None
    lib().oracle_conv_k(n, c_in, c_out, h, w, ksize, stride, _p(x), _p(wd), _p(b), int(relu), _p(y), _p(pre), _p(sc),
                        threads or default_threads())
    if want_pre or want_scale:
        return y, pre, sc
    return y


def conv_k_at(x, wd, pts, stride=1, bias=None, relu=False, threads=None):
    """Reference result at sampled outputs of the convolution's own output grid.  Returns (y, pre, scale)."""
    assert x.dtype in (np.float32, np.float16) and x.flags.c_contiguous
    wd = _c(wd, np.float64)
    n, c_in, h, w = x.shape
    c_out, _, ksize, _ = wd.shape
    pts = _c(pts, np.int32)
    npts = pts.shape[0]
    b = None if bias is None else _c(bias, np.float64)
    y = np.empty(npts, dtype=np.float64)
    pre = np.empty(npts, dtype=np.float64)
    sc = np.empty(npts, dtype=np.float64)
    lib().oracle_conv_k_at(n, c_in, c_out, h, w, ksize, stride, _p(wd), _p(b), int(relu), int(x.dtype == np.float16),
                           _p(x), npts, _p(pts), _p(y), _p(pre), _p(sc), threads or default_threads())
    return y, pre, sc


def brute_k(x, ksize, stride, taps, masks, pattern_id, conn, weights, c_out, bias=None, relu=False):
    x = _c(x, np.float64)
    n, c_in, h, w = x.shape
    masks = _c(masks, np.uint64)
    pid = _c(pattern_id, np.int32)
    cm = _c(conn, np.uint8)
    wt = _c(weights, np.float64).reshape(-1)
    b = None if bias is None else _c(bias, np.float64)
    y = np.empty((n, c_out, out_size(h, stride), out_size(w, stride)), dtype=np.float64)
    lib().oracle_brute_k(n, c_in, c_out, h, w, ksize, stride, taps, _p(masks), _p(pid), _p(cm), _p(wt), _p(x), _p(b),
                         int(relu), _p(y))
    return y


# -- conveniences over a synthetic layer description (duck-typed: any object with the
#    fields of synth.Layer) ---------------------------------------------------------

def layer_dense_weights(layer) -> np.ndarray:
    """Wd of a layer, with the weights first rounded to binary16 when the layer stores fp16."""
    w = np.asarray(layer.weights, dtype=np.float64)
    if layer.dtype == "f16":
        w = widen_f16(round_f16(w))
    ksize = getattr(layer, "ksize", 3)
    if ksize != 3 or (not layer.dense and layer.taps != 4):
        return expand_weights_k(layer.c_in, layer.c_out, ksize, layer.pattern_masks, layer.pattern_id, layer.conn_mask,
                                w, taps=layer.taps)
    return expand_weights(layer.c_in, layer.c_out, layer.pattern_masks, layer.pattern_id, layer.conn_mask, w,
                          taps=9 if layer.dense else 4)


def layer_reference(layer, x, relu=None, threads=None):
    """(y, pre, scale) of the whole layer on input x (already in the storage dtype).  For a layer with
    a fused 2x2 max-pool y and scale are pooled; pre stays the convolution's own (it only sets the
    error measure's floor)."""
    wd = layer_dense_weights(layer)
    relu = layer.relu if relu is None else relu
    stride, pool = getattr(layer, "stride", 1), getattr(layer, "pool", False)
    if wd.shape[-1] == 3 and stride == 1:
        y, pre, sc = conv(np.asarray(x, dtype=np.float64), wd, layer.bias, relu, want_pre=True, want_scale=True,
                          threads=threads)
    else:
        y, pre, sc = conv_k(np.asarray(x, dtype=np.float64), wd, stride, layer.bias, relu, want_pre=True,
                            want_scale=True, threads=threads)
    if pool:
        y, sc = maxpool2(y), maxpool2(sc)
    return y, pre, sc


# ---- block-pruned matrix product (section 2.1.2) ----

def block_expand(m, k, bm, bk, row_keep, col_keep, weights) -> np.ndarray:
    """Masked dense matrix Wd [m, k] in float64."""
    rk, ck, w = _c(row_keep, np.uint8), _c(col_keep, np.uint8), _c(weights, np.float64)
    blocks = ((m + bm - 1) // bm) * ((k + bk - 1) // bk)
    assert rk.size == blocks * bm and ck.size == blocks * bk and w.shape == (m, k)
    wd = np.empty((m, k), dtype=np.float64)
    if lib().oracle_block_expand(m, k, bm, bk, _p(rk), _p(ck), _p(w), _p(wd)) != 0:
        raise ValueError("bad block layer shape")
    return wd


def gemm(wd, x, bias=None, relu=False, want_pre=False, want_scale=False, threads=None):
    """y = act(wd @ x + bias) by three plain loops in float64; x is [k, n]."""
    wd, x = _c(wd, np.float64), _c(x, np.float64)
    m, k = wd.shape
    assert x.shape[0] == k
    n = x.shape[1]
    b = None if bias is None else _c(bias, np.float64)
    y = np.empty((m, n), dtype=np.float64)
    pre = np.empty((m, n), dtype=np.float64) if want_pre else None
    sc = np.empty((m, n), dtype=np.float64) if want_scale else None
    lib().oracle_gemm(m, k, n, _p(wd), _p(x), _p(b), int(relu), _p(y), _p(pre), _p(sc), threads or default_threads())
    out = (y,)
    if want_pre:
        out += (pre,)
    if want_scale:
        out += (sc,)
    return out if len(out) > 1 else y


def gemm_at(wd, x, pts, bias=None, relu=False, threads=None):
    """(y, pre, scale) at the (row, column) pairs pts [count, 2]."""
    wd, x = _c(wd, np.float64), _c(x, np.float64)
    m, k = wd.shape
    n = x.shape[1]
    pts = _c(pts, np.int32)
    assert pts.ndim == 2 and pts.shape[1] == 2 and pts[:, 0].max(initial=0) < m and pts[:, 1].max(initial=0) < n and pts.min(initial=0) >= 0
    b = None if bias is None else _c(bias, np.float64)
    cnt = pts.shape[0]
    y, pre, sc = (np.empty(cnt, dtype=np.float64) for _ in range(3))
    lib().oracle_gemm_at(m, k, n, _p(wd), _p(x), _p(b), int(relu), _p(pts), cnt, _p(y), _p(pre), _p(sc), threads or default_threads())
    return y, pre, sc


def block_brute(m, k, bm, bk, row_keep, col_keep, weights, x, bias=None, relu=False) -> np.ndarray:
    """Gather-style evaluation that never forms the masked matrix (a pin for block_expand + gemm)."""
    rk, ck, w, x = _c(row_keep, np.uint8), _c(col_keep, np.uint8), _c(weights, np.float64), _c(x, np.float64)
    n = x.shape[1]
    b = None if bias is None else _c(bias, np.float64)
    y = np.empty((m, n), dtype=np.float64)
    lib().oracle_block_brute(m, k, n, bm, bk, _p(rk), _p(ck), _p(w), _p(x), _p(b), int(relu), _p(y))
    return y


def block_layer_reference(layer, x, relu=None, threads=None):
    """(y, pre, scale) of a synth.BlockLayer on x [k, n]; weights, input and bias are taken as stored
    (binary16-rounded first when the layer's storage type is f16)."""
    w = layer.weights.astype(np.float64)
    if layer.dtype == "f16":
        w = widen_f16(round_f16(w))
    wd = block_expand(layer.m, layer.k, layer.bm, layer.bk, layer.row_keep, layer.col_keep, w)
    return gemm(wd, np.asarray(x, dtype=np.float64), layer.bias, layer.relu if relu is None else relu, True, True, threads)


# ---- deep reuse (section 2.3.2) ----

def reuse_signatures(x, hyperplanes, seg_len, hash_bits) -> np.ndarray:
    """uint16 [n, k // seg_len]: sign-random-projection signature of every neuron vector (binary32, fixed order)."""
    x, hp = _c(x, np.float32), _c(hyperplanes, np.float32)
    n, k = x.shape
    assert k % seg_len == 0 and hp.size == (k // seg_len) * hash_bits * seg_len
    sig = np.empty((n, k // seg_len), dtype=np.uint16)
    if lib().oracle_reuse_signatures(n, k, seg_len, hash_bits, _p(x), _p(hp), _p(sig)) != 0:
        raise ValueError("bad deep-reuse shape")
    return sig


def reuse_representatives(sig, hash_bits) -> np.ndarray:
    """int32 [S, 2**hash_bits]: lowest row index per cluster, -1 where empty."""
    sig = _c(sig, np.uint16)
    n, S = sig.shape
    rep = np.empty((S, 1 << hash_bits), dtype=np.int32)
    lib().oracle_reuse_representatives(n, S, hash_bits, _p(sig), _p(rep))
    return rep


def reuse_layer(x, w, hyperplanes, seg_len, hash_bits, bias=None, relu=False):
    """(y, pre, scale, sig, rep) of the deep-reuse approximation of act(x @ w + bias); x [n, k] float32 values."""
    sig = reuse_signatures(x, hyperplanes, seg_len, hash_bits)
    rep = reuse_representatives(sig, hash_bits)
    x64, w64 = _c(x, np.float64), _c(w, np.float64)
    n, k = x64.shape
    m = w64.shape[1]
    assert w64.shape[0] == k
    b = None if bias is None else _c(bias, np.float64)
    y, pre, sc = (np.empty((n, m), dtype=np.float64) for _ in range(3))
    lib().oracle_reuse_apply(n, k, m, seg_len, hash_bits, _p(x64), _p(w64), _p(b), _p(sig), _p(rep), int(relu), _p(y), _p(pre), _p(sc))
    return y, pre, sc, sig, rep
