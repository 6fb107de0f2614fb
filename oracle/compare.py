"""Error measures used when a GPU result is compared with the checker's (test infrastructure)."""
from __future__ import annotations

import numpy as np

TOL = {"f32": 1e-5, "f16": 2e-3}


def error_report(got, ref_y, ref_pre, ref_scale=None) -> dict:
    """got, ref_y: same shape.  The gate is E = max |got - ref| / max(|ref|, sigma), sigma = RMS of the
    reference pre-activation values: a relative error whose denominator is floored at the typical
    output magnitude, since outputs near zero (cancellation, ReLU) have no meaningful relative error.
    Also returns the error relative to the per-output magnitude sum(|w||x|) and the normwise error."""
    got = np.asarray(got, dtype=np.float64)
    ref_y = np.asarray(ref_y, dtype=np.float64)
    sigma = float(np.sqrt(np.mean(np.asarray(ref_pre, dtype=np.float64) ** 2)))
    diff = np.abs(got - ref_y)
    denom = np.maximum(np.abs(ref_y), sigma if sigma > 0 else 1.0)
    rep = {"E": float(np.max(diff / denom)) if diff.size else 0.0, "sigma": sigma,
           "max_abs": float(diff.max()) if diff.size else 0.0,
           "normwise": float(np.linalg.norm(diff.ravel()) / max(np.linalg.norm(ref_y.ravel()), 1e-300))}
    if ref_scale is not None:
        s = np.maximum(np.asarray(ref_scale, dtype=np.float64), 1e-300)
        rep["E_scale"] = float(np.max(diff / s)) if diff.size else 0.0
    return rep


def sample_points(n, c_out, h, w, count, seed=0):
    """Sampled output coordinates: random ones plus corners, edges and the last element."""
    rs = np.random.RandomState(seed)
    pts = np.stack([rs.randint(0, n, count), rs.randint(0, c_out, count), rs.randint(0, h, count),
                    rs.randint(0, w, count)], axis=1)
    fixed = []
    for img in (0, n - 1):
        for co in (0, c_out - 1):
            for oy in (0, h // 2, h - 1):
                for ox in (0, w // 2, w - 1):
                    fixed.append((img, co, oy, ox))
    return np.concatenate([pts, np.array(fixed)], axis=0).astype(np.int32)
