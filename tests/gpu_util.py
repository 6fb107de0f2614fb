"""Helpers for the GPU parity tests: run a layer through the C-ABI library and compare with the CPU checker."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from oracle.compare import TOL, error_report, sample_points, structured_points
import paper_2206_10620_amd as pp

FULL_LIMIT = 3.0e9      # dense multiply-accumulates above which the checker is evaluated at sampled outputs only


def to_device(x_np):
    return torch.from_numpy(np.ascontiguousarray(x_np)).cuda()


def run_layer(lay, x_np, tuning=None, relu=None, n_hint=None):
    """One forward pass on the GPU; returns (y as numpy in the storage dtype, chosen parameters)."""
    if relu is not None and relu != lay.relu:
        import copy
        lay = copy.copy(lay)
        lay.relu = relu
    plan = pp.plan_from_layer(lay, tuning=tuning, n_hint=n_hint if n_hint is not None else x_np.shape[0])
    try:
        xd = to_device(x_np)
        yd = torch.full((x_np.shape[0], lay.c_out, plan.out_h, plan.out_w), float("nan"), dtype=xd.dtype, device="cuda")
        plan.run(xd, yd)
        torch.cuda.synchronize()
        return yd.cpu().numpy(), plan.query()["chosen"]
    finally:
        plan.close()


def reference_at(lay, x_np, wd, pts, relu_flag):
    """Checker values at sampled stored outputs pts (n, co, y, x of the stored grid).  With a fused pool a
    stored output is the maximum of four activated convolution outputs."""
    ksize, stride, pool = getattr(lay, "ksize", 3), getattr(lay, "stride", 1), getattr(lay, "pool", False)
    x_np = np.ascontiguousarray(x_np)
    if not pool:
        if ksize == 3 and stride == 1:
            return oracle.conv_at(x_np, wd, pts, lay.bias, relu_flag)
        return oracle.conv_k_at(x_np, wd, pts, stride, lay.bias, relu_flag)
    quad = np.repeat(pts, 4, axis=0)
    quad[:, 2] = 2 * quad[:, 2] + np.tile([0, 0, 1, 1], len(pts))
    quad[:, 3] = 2 * quad[:, 3] + np.tile([0, 1, 0, 1], len(pts))
    y4, pre4, sc4 = oracle.conv_k_at(x_np, wd, quad.astype(np.int32), stride, lay.bias, relu_flag)
    return y4.reshape(-1, 4).max(axis=1), pre4, sc4.reshape(-1, 4).max(axis=1)


def tile_boundary_points(lay, n, chosen):
    """Stored-output coordinates on both sides of every tile boundary of the plan that ran (row bands of
    the batch as one tall image, column strips), on the first and last row of every image and over the
    whole last ragged tile: the places a sampled comparison of a large layer would otherwise only hit by
    luck.  The tile geometry is read from the plan's reported parameters."""
    pool = 2 if getattr(lay, "pool", False) else 1
    if chosen["variant"] == 3:
        band, strip = max(chosen["tile_rows"] // pool, 1), max(chosen["tile_cols"] // pool, 1)
        # rows per image of the tall image: the general kernel pads by the kernel's reach, the direct one by one row
        rpi = lay.out_h + 1
    elif chosen["variant"] == 2:
        band, strip = chosen["rows_per_lane"] * max(64 // chosen["lanes_x"], 1), 4 * chosen["lanes_x"]
        rpi = lay.out_h + 1
    else:
        band, strip, rpi = 1, 256, lay.out_h
    return structured_points(n, lay.c_out, lay.out_h, lay.out_w, band, strip, rpi, seed=lay.seed)


def check_layer(lay, x_np=None, tuning=None, relu=None, tol=None, points=4096, label="", extra_points=None, n_hint=None):
    """Compare GPU output with the checker: every element when the layer is small, sampled outputs otherwise
    (random ones, corners and edges, plus extra_points: an int array [k, 4] of stored-output coordinates)."""
    if x_np is None:
        x_np = lay.make_input()
    relu_flag = lay.relu if relu is None else relu
    y, chosen = run_layer(lay, x_np, tuning, relu, n_hint)
    assert not np.isnan(y.astype(np.float32)).any(), f"{label}: output has unwritten (NaN) elements"
    n = x_np.shape[0]
    ksize = getattr(lay, "ksize", 3)
    dense_macs = float(ksize * ksize) * n * lay.conv_h * lay.conv_w * lay.c_in * lay.c_out
    assert y.shape == (n, lay.c_out, lay.out_h, lay.out_w), (y.shape, label)
    if dense_macs <= FULL_LIMIT:
        ref, pre, scale = oracle.layer_reference(lay, x_np.astype(np.float64), relu=relu_flag)
        rep = error_report(y, ref, pre, scale)
    else:
        wd = oracle.layer_dense_weights(lay)
        pts = sample_points(n, lay.c_out, lay.out_h, lay.out_w, points, seed=lay.seed)
        pts = np.concatenate([pts, tile_boundary_points(lay, n, chosen)], axis=0)
        if extra_points is not None and len(extra_points):
            pts = np.concatenate([pts, np.asarray(extra_points, dtype=np.int32)], axis=0)
        ref, pre, scale = reference_at(lay, x_np, wd, pts, relu_flag)
        got = y[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]]
        rep = error_report(got, ref, pre, scale)
    rep["chosen"] = chosen
    tol = TOL[lay.dtype] if tol is None else tol
    assert rep["E"] <= tol, f"{label} {lay.name}: E={rep['E']:.3e} > {tol:g}  ({rep})"
    return rep, y
