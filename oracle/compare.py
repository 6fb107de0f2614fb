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


def structured_points(n, c_out, h, w, band_rows, strip_cols, rows_per_image, count_cap=6000, filters=None, seed=0):
    """Sampled output coordinates placed where a tiled kernel can go wrong without a random sample noticing:
    both sides of every boundary between row bands (band_rows rows of the batch laid out as one tall image
    with rows_per_image rows per image: h plus separator rows) and between column strips (strip_cols columns),
    rows 0 and h - 1 of every image, and the whole of the last (ragged) band x strip tile.  The geometry comes
    in as plain numbers (the test reads them from the plan it checks).  At most about count_cap points, drawn
    with a seeded generator when a category has more; each point is paired with a filter from `filters`
    (default: first, last, and both sides of every multiple of 64)."""
    rs = np.random.RandomState(seed)
    if filters is None:
        fs = {0, c_out - 1}
        for b in range(64, c_out, 64):
            fs.update((b - 1, b))
        filters = sorted(f for f in fs if 0 <= f < c_out)
    filters = np.asarray(filters, dtype=np.int64)
    cols_edge = sorted({x for k in range(1, (w + strip_cols - 1) // strip_cols) for x in (k * strip_cols - 1, k * strip_cols) if 0 <= x < w} | {0, w - 1})
    vrows = n * rows_per_image - (rows_per_image - h)
    rows_edge = set()
    for k in range(1, (vrows + band_rows - 1) // band_rows):
        rows_edge.update((k * band_rows - 1, k * band_rows))
    for img in range(n):
        rows_edge.update((img * rows_per_image, img * rows_per_image + h - 1))
    rows_edge = sorted(v for v in rows_edge if 0 <= v < vrows and v % rows_per_image < h)

    def pick(seq, k):
        seq = list(seq)
        if len(seq) <= k:
            return seq
        idx = rs.choice(len(seq), size=k, replace=False)
        return [seq[i] for i in sorted(idx)]

    pts = []
    cap = max(count_cap // 4, 16)
    some_cols = pick(range(w), 8) + cols_edge[:2] + cols_edge[-2:]
    for v in pick(rows_edge, max(cap // max(len(some_cols), 1), 1)):          # band boundaries and image edges x some columns
        for x in some_cols:
            pts.append((v, x))
    some_rows = pick([v for v in range(vrows) if v % rows_per_image < h], 8)
    for x in pick(cols_edge, max(cap // 8, 1)):                                # strip boundaries x some rows
        for v in some_rows:
            pts.append((v, x))
    for v in pick(rows_edge, 64):                                               # crossings of the two
        for x in pick(cols_edge, 16):
            pts.append((v, x))
    last_v0 = ((vrows - 1) // band_rows) * band_rows
    last_x0 = ((w - 1) // strip_cols) * strip_cols
    last_tile = [(v, x) for v in range(last_v0, vrows) if v % rows_per_image < h for x in range(last_x0, w)]
    pts.extend(pick(last_tile, cap))                                           # the last ragged tile
    pts = sorted(set(pts))
    out = np.empty((len(pts), 4), dtype=np.int32)
    for i, (v, x) in enumerate(pts):
        out[i] = (v // rows_per_image, int(filters[rs.randint(len(filters))]), v % rows_per_image, x)
    return out
