"""Helpers for the GPU parity tests: run a layer through the C-ABI library and compare with the CPU checker."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from oracle.compare import TOL, error_report, sample_points
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
        yd = torch.full((x_np.shape[0], lay.c_out, lay.h, lay.w), float("nan"), dtype=xd.dtype, device="cuda")
        plan.run(xd, yd)
        torch.cuda.synchronize()
        return yd.cpu().numpy(), plan.query()["chosen"]
    finally:
        plan.close()


def check_layer(lay, x_np=None, tuning=None, relu=None, tol=None, points=4096, label=""):
    """Compare GPU output with the checker: every element when the layer is small, sampled outputs otherwise."""
    if x_np is None:
        x_np = lay.make_input()
    relu_flag = lay.relu if relu is None else relu
    y, chosen = run_layer(lay, x_np, tuning, relu)
    assert not np.isnan(y.astype(np.float32)).any(), f"{label}: output has unwritten (NaN) elements"
    n = x_np.shape[0]
    dense_macs = 9.0 * n * lay.h * lay.w * lay.c_in * lay.c_out
    wd = oracle.layer_dense_weights(lay)
    if dense_macs <= FULL_LIMIT:
        ref, pre, scale = oracle.conv(x_np.astype(np.float64), wd, lay.bias, relu_flag, want_pre=True, want_scale=True)
        rep = error_report(y, ref, pre, scale)
    else:
        pts = sample_points(n, lay.c_out, lay.h, lay.w, points, seed=lay.seed)
        ref, pre, scale = oracle.conv_at(np.ascontiguousarray(x_np), wd, pts, lay.bias, relu_flag)
        got = y[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]]
        rep = error_report(got, ref, pre, scale)
    rep["chosen"] = chosen
    tol = TOL[lay.dtype] if tol is None else tol
    assert rep["E"] <= tol, f"{label} {lay.name}: E={rep['E']:.3e} > {tol:g}  ({rep})"
    return rep, y
