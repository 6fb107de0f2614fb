"""Pins for the CPU checker: each test ties oracle/ to something other than itself
(a hand-worked example, a closed form, a library routine, a brute-force gather)."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_layer(seed, n=2, c_in=3, c_out=4, h=5, w=4, keep=0.6, pset=synth.PSET8, bias=True):
    lay = synth.random_pruned_layer("tiny", n, c_in, c_out, h, w, "f32", pset, keep, 0.5, seed, with_bias=bias)
    x = lay.make_input().astype(np.float64)
    return lay, x


def numpy_dense_weights(lay):
    """Independent construction of the masked dense weights (numpy, from the tap lists)."""
    wd = np.zeros((lay.c_out, lay.c_in, 3, 3))
    for k in range(lay.c_out * lay.c_in):
        if not lay.conn_mask[k]:
            continue
        co, ci = divmod(k, lay.c_in)
        if lay.dense:
            wd[co, ci] = lay.weights[k].reshape(3, 3)
            continue
        for j, t in enumerate(synth.mask_taps(lay.pattern_masks[lay.pattern_id[k]])):
            wd[co, ci, t // 3, t % 3] = lay.weights[k, j]
    return wd


def test_hand_worked_example():
    g = json.load(open(os.path.join(GOLDEN, "hand_conv_3x3.json")))
    wd = oracle.expand_weights(g["c_in"], g["c_out"], g["pattern_masks"], g["pattern_id"], g["conn_mask"],
                               np.array(g["weights"], dtype=np.float64))
    x = np.array(g["x"], dtype=np.float64)[None]
    y = oracle.conv(x, wd, np.array(g["bias"]), relu=False)
    assert np.array_equal(y[0], np.array(g["y"], dtype=np.float64))
    yb = oracle.brute(x, g["pattern_masks"], g["pattern_id"], g["conn_mask"], np.array(g["weights"], dtype=np.float64),
                      g["c_out"], np.array(g["bias"]))
    assert np.array_equal(yb[0], np.array(g["y"], dtype=np.float64))
    pts = np.array([[0, co, oy, ox] for co in range(2) for oy in range(3) for ox in range(3)], dtype=np.int32)
    ya, _, _ = oracle.conv_at(x.astype(np.float32), wd, pts, np.array(g["bias"]))
    assert np.array_equal(ya.reshape(2, 3, 3), np.array(g["y"], dtype=np.float64))


@pytest.mark.parametrize("shape", [(2, 3, 4, 5, 4), (1, 2, 3, 1, 1), (1, 5, 2, 1, 7), (3, 1, 1, 6, 1), (1, 8, 6, 7, 9)])
@pytest.mark.parametrize("relu", [False, True])
def test_brute_force_gather(shape, relu):
    n, c_in, c_out, h, w = shape
    for seed in (0, 1):
        for pset in (synth.PSET8, synth.PSET16):
            lay, x = tiny_layer(seed, n, c_in, c_out, h, w, pset=pset)
            wd = oracle.layer_dense_weights(lay)
            y = oracle.conv(x, wd, lay.bias, relu)
            yb = oracle.brute(x, lay.pattern_masks, lay.pattern_id, lay.conn_mask, lay.weights, c_out, lay.bias, relu)
            assert np.max(np.abs(y - yb)) <= 1e-13 * max(1.0, np.max(np.abs(yb)))


@pytest.mark.parametrize("seed", [0, 3])
def test_library_conv_float64(seed):
    """A masked dense conv is a dense conv: torch's float64 CPU conv2d on independently built weights."""
    lay, x = tiny_layer(seed, 2, 6, 5, 9, 11)
    wd = numpy_dense_weights(lay)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(wd), torch.from_numpy(lay.bias.astype(np.float64)),
                                     stride=1, padding=1).numpy()
    y, pre, scale = oracle.layer_reference(lay, x, relu=False)
    assert np.max(np.abs(y - ref)) < 1e-12
    assert np.array_equal(y, pre)
    yr = oracle.layer_reference(lay, x, relu=True)[0]
    assert np.max(np.abs(yr - np.maximum(ref, 0))) < 1e-12
    # the error scale is the same sum with absolute values
    sref = torch.nn.functional.conv2d(torch.from_numpy(np.abs(x)), torch.from_numpy(np.abs(wd)),
                                      torch.from_numpy(np.abs(lay.bias.astype(np.float64))), padding=1).numpy()
    assert np.max(np.abs(scale - sref)) < 1e-12


def test_all_taps_all_kernels_is_dense_conv():
    lay = synth.dense_layer("dense", 2, 3, 4, 6, 5, "f32", 0.3, 7)
    x = lay.make_input().astype(np.float64)
    w9 = lay.weights.astype(np.float64).reshape(lay.c_out, lay.c_in, 3, 3)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w9),
                                     torch.from_numpy(lay.bias.astype(np.float64)), padding=1).numpy()
    y = oracle.layer_reference(lay, x, relu=False)[0]
    assert np.max(np.abs(y - ref)) < 1e-12


@pytest.mark.parametrize("relu", [False, True])
def test_empty_mask_gives_bias(relu):
    lay, x = tiny_layer(2)
    lay.conn_mask[:] = 0
    y = oracle.layer_reference(lay, x, relu=relu)[0]
    b = lay.bias.astype(np.float64)
    want = np.maximum(b, 0) if relu else b
    assert np.array_equal(y, np.broadcast_to(want[None, :, None, None], y.shape))


def test_impulse_response_closed_form():
    """x = delta at (ci0, y0, x0): output (y0-dy, x0-dx) of filter co equals the weight of tap (dy, dx)
    of kernel (co, ci0), everything else is zero.  Fixes tap orientation (no kernel flip) and padding."""
    lay, _ = tiny_layer(5, n=1, c_in=3, c_out=4, h=5, w=6, keep=0.8, bias=False)
    wd = oracle.layer_dense_weights(lay)
    for (ci0, y0, x0) in [(0, 2, 3), (1, 0, 0), (2, 4, 5), (1, 0, 5)]:
        x = np.zeros((1, 3, 5, 6))
        x[0, ci0, y0, x0] = 1.0
        y = oracle.conv(x, wd)
        want = np.zeros_like(y)
        for co in range(4):
            k = co * 3 + ci0
            if not lay.conn_mask[k]:
                continue
            for j, t in enumerate(synth.mask_taps(lay.pattern_masks[lay.pattern_id[k]])):
                dy, dx = t // 3 - 1, t % 3 - 1
                oy, ox = y0 - dy, x0 - dx
                if 0 <= oy < 5 and 0 <= ox < 6:
                    want[0, co, oy, ox] = lay.weights[k, j]
        assert np.array_equal(y, want)


def test_constant_input_closed_form():
    """x = 1: interior outputs are bias + sum of all kept weights of the filter (independent of where
    the taps sit); the top-left corner drops exactly the taps with dy = -1 or dx = -1."""
    lay, _ = tiny_layer(11, n=1, c_in=5, c_out=6, h=6, w=7)
    x = np.ones((1, 5, 6, 7))
    y = oracle.layer_reference(lay, x, relu=False)[0]
    wts = lay.weights.astype(np.float64).reshape(6, 5, 4) * lay.conn_mask.reshape(6, 5, 1)
    interior = lay.bias + wts.sum(axis=(1, 2))
    assert np.max(np.abs(y[0, :, 1:-1, 1:-1] - interior[:, None, None])) < 1e-13
    corner = lay.bias.astype(np.float64).copy()
    for k in range(30):
        if lay.conn_mask[k]:
            for j, t in enumerate(synth.mask_taps(lay.pattern_masks[lay.pattern_id[k]])):
                if t // 3 >= 1 and t % 3 >= 1:
                    corner[k // 5] += float(lay.weights[k, j])
    assert np.max(np.abs(y[0, :, 0, 0] - corner)) < 1e-13


def test_linearity_in_input_and_weights():
    lay, x1 = tiny_layer(4, bias=False)
    x2 = np.cos(np.arange(x1.size, dtype=np.float64)).reshape(x1.shape)
    wd = oracle.layer_dense_weights(lay)
    a, b = 0.75, -2.0   # exactly representable scalings
    lhs = oracle.conv(a * x1 + b * x2, wd)
    rhs = a * oracle.conv(x1, wd) + b * oracle.conv(x2, wd)
    assert np.max(np.abs(lhs - rhs)) < 1e-12
    assert np.max(np.abs(oracle.conv(x1, 4.0 * wd) - 4.0 * oracle.conv(x1, wd))) == 0.0


def test_centre_only_is_matrix_product():
    """Every PSET8 pattern holds the centre tap; with the other three weights zero the layer is a 1x1
    convolution, i.e. Wc [c_out x c_in] times x [c_in x (h*w)]."""
    lay, x = tiny_layer(8, n=2, c_in=7, c_out=5, h=4, w=6, bias=False)
    wc = np.zeros((5, 7))
    for k in range(35):
        taps = synth.mask_taps(lay.pattern_masks[lay.pattern_id[k]])
        j = taps.index(4)
        keepw = lay.weights[k, j]
        lay.weights[k, :] = 0
        lay.weights[k, j] = keepw
        if lay.conn_mask[k]:
            wc[k // 7, k % 7] = keepw
    y = oracle.layer_reference(lay, x, relu=False)[0]
    want = np.einsum("oc,nchw->nohw", wc, x)
    assert np.max(np.abs(y - want)) < 1e-13


def test_filter_permutation_equivariance():
    lay, x = tiny_layer(9, c_in=4, c_out=6)
    y = oracle.layer_reference(lay, x)[0]
    perm = np.array([3, 0, 5, 1, 4, 2])
    rows = (perm[:, None] * lay.c_in + np.arange(lay.c_in)[None, :]).reshape(-1)
    lay2 = synth.Layer("p", lay.n, lay.c_in, lay.c_out, lay.h, lay.w, "f32", lay.pattern_masks, lay.pattern_id[rows],
                       lay.conn_mask[rows], lay.weights[rows], lay.bias[perm], relu=lay.relu)
    y2 = oracle.layer_reference(lay2, x)[0]
    assert np.array_equal(y2, y[:, perm])


def test_sampled_points_match_full_tensor():
    lay, x = tiny_layer(6, n=2, c_in=5, c_out=4, h=7, w=5)
    for dt in (np.float32, np.float16):
        xs = np.ascontiguousarray(x.astype(dt))
        y, pre, scale = oracle.layer_reference(lay, xs.astype(np.float64))
        idx = np.stack(np.unravel_index(np.arange(y.size), y.shape), axis=1).astype(np.int32)
        ya, prea, sa = oracle.conv_at(xs, oracle.layer_dense_weights(lay), idx, lay.bias, lay.relu)
        assert np.array_equal(ya.reshape(y.shape), y)
        assert np.array_equal(prea.reshape(y.shape), pre)
        assert np.array_equal(sa.reshape(y.shape), scale)


def test_binary16_rounding_against_numpy():
    rs = np.random.RandomState(0)
    v = np.concatenate([
        rs.standard_normal(20000), rs.standard_normal(2000) * 1e-6, rs.standard_normal(2000) * 1e4,
        np.array([0.0, -0.0, 1.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25,
                  2.0 ** -14, 2.0 ** -14 - 2.0 ** -26, 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 1 + 2.0 ** -11 + 2.0 ** -30,
                  2047.5, 2048.5, 2049.5]),
    ])
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    got = oracle.round_f16(v)
    assert np.array_equal(got, want)
    allbits = np.arange(65536, dtype=np.uint16)
    wide = oracle.widen_f16(allbits)
    ref = allbits.view(np.float16).astype(np.float64)
    assert np.array_equal(np.isnan(wide), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(wide[ok], ref[ok])
    # ties go to the even neighbour: 1 + 2^-11 -> 1, 1 + 3*2^-11 -> 1 + 2^-9
    assert oracle.widen_f16(oracle.round_f16(np.array([1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11]))).tolist() == [1.0, 1 + 2.0 ** -9]


def test_fp16_layer_uses_rounded_weights():
    lay, x = tiny_layer(12)
    lay.dtype = "f16"
    wd = oracle.layer_dense_weights(lay)
    w16 = lay.weights.astype(np.float16).astype(np.float64)
    lay32 = synth.Layer("w", lay.n, lay.c_in, lay.c_out, lay.h, lay.w, "f32", lay.pattern_masks, lay.pattern_id,
                        lay.conn_mask, w16, lay.bias)
    assert np.array_equal(wd, numpy_dense_weights(lay32))


def test_maxpool_against_library():
    x = np.random.RandomState(1).standard_normal((2, 3, 6, 8))
    want = torch.nn.functional.max_pool2d(torch.from_numpy(x), 2).numpy()
    assert np.array_equal(oracle.maxpool2(x), want)


def test_invalid_descriptions_are_rejected():
    with pytest.raises(ValueError):
        oracle.expand_weights(1, 1, [0x1FF], [0], [1], np.zeros(4))          # five or more taps in a 4-entry pattern
    with pytest.raises(ValueError):
        oracle.expand_weights(1, 1, [0x03A], [1], [1], np.zeros(4))          # pattern id out of range


# ---- reference filter-kernel ordering -------------------------------------------------

def test_plan_hand_worked_example():
    g = json.load(open(os.path.join(GOLDEN, "hand_plan_4x4.json")))
    r = oracle.plan_ref(g["c_in"], g["c_out"], g["num_patterns"], np.maximum(g["pattern_id"], 0), g["conn_mask"])
    assert r["perm"].tolist() == g["perm"]
    assert r["kcount"].tolist() == g["kcount"]
    assert r["pat_off"].tolist() == g["pat_off"]
    assert r["kidx"].tolist() == g["kidx"]
    assert r["kpat"].tolist() == g["kpat"]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_plan_structural_invariants(seed):
    lay = synth.random_pruned_layer("p", 1, 24, 40, 4, 4, "f32", synth.PSET16, 0.37, 0.1, seed)
    lay.conn_mask.reshape(40, 24)[5] = 0          # an empty filter
    lay.conn_mask.reshape(40, 24)[9] = 1          # a full one
    p = len(lay.pattern_masks)
    r = oracle.plan_ref(lay.c_in, lay.c_out, p, lay.pattern_id, lay.conn_mask)
    assert sorted(r["perm"].tolist()) == list(range(40))
    assert r["kcount"].sum() == r["k_kept"] == np.count_nonzero(lay.conn_mask)
    assert np.all(np.diff(r["kcount"]) <= 0)
    assert r["perm"][0] == 9 and r["perm"][-1] == 5
    assert np.all(np.diff(r["pat_off"], axis=1) >= 0) and np.array_equal(r["pat_off"][:, -1], r["kcount"])
    start = 0
    wd = np.zeros((40, 24, 3, 3))
    for pos in range(40):
        co, cnt = r["perm"][pos], r["kcount"][pos]
        keys = [(int(r["kpat"][start + i]), int(r["kidx"][start + i])) for i in range(cnt)]
        assert keys == sorted(set(keys))                                  # strictly increasing (pattern, channel)
        for q in range(p):
            seg = r["kpat"][start + r["pat_off"][pos, q]: start + r["pat_off"][pos, q + 1]]
            assert np.all(seg == q)
        for i in range(cnt):
            ci = r["kidx"][start + i]
            assert lay.conn_mask[co * 24 + ci] and lay.pattern_id[co * 24 + ci] == r["kpat"][start + i]
            assert r["wsel"][start + i] == co * 24 + ci
            for j, t in enumerate(synth.mask_taps(lay.pattern_masks[r["kpat"][start + i]])):
                wd[co, ci, t // 3, t % 3] = lay.weights[r["wsel"][start + i], j]
        start += cnt
    # scattering the reordered kernels back reproduces the masked dense weights
    assert np.array_equal(wd, oracle.layer_dense_weights(lay))
    # between equal-count neighbours the histogram is non-increasing lexicographically
    hist = np.diff(r["pat_off"], axis=1)
    for pos in range(39):
        if r["kcount"][pos] == r["kcount"][pos + 1]:
            a, b = hist[pos].tolist(), hist[pos + 1].tolist()
            assert a > b or (a == b and r["perm"][pos] < r["perm"][pos + 1])


# ---- the comparison helpers (oracle/compare.py) ------------------------------------------------

def test_error_report_on_hand_made_arrays():
    """E = max |got - ref| / max(|ref|, sigma) with sigma = RMS of the pre-activations, worked by hand."""
    from oracle.compare import error_report
    pre = np.array([3.0, -4.0, 0.0, 0.0])                    # sigma = sqrt((9 + 16) / 4) = 2.5
    ref = np.maximum(pre, 0.0)                               # ReLU: [3, 0, 0, 0]
    got = np.array([3.3, 0.05, 0.0, -0.25])
    rep = error_report(got, ref, pre, np.array([10.0, 10.0, 1.0, 0.5]))
    assert rep["sigma"] == pytest.approx(2.5)
    # element errors 0.3, 0.05, 0, 0.25 over denominators max(3, 2.5), 2.5, 2.5, 2.5
    assert rep["E"] == pytest.approx(max(0.3 / 3.0, 0.05 / 2.5, 0.25 / 2.5))
    assert rep["max_abs"] == pytest.approx(0.3)
    assert rep["E_scale"] == pytest.approx(0.25 / 0.5)
    assert rep["normwise"] == pytest.approx(np.sqrt(0.3 ** 2 + 0.05 ** 2 + 0.25 ** 2) / 3.0)
    # the floor: an output near zero is measured against sigma, not against itself
    rep = error_report(np.array([1e-9]), np.array([0.0]), np.array([2.0]))
    assert rep["E"] == pytest.approx(1e-9 / 2.0)
    # above the floor it is the plain relative error
    rep = error_report(np.array([101.0, 0.0]), np.array([100.0, 0.0]), np.array([100.0, 0.0]))
    assert rep["E"] == pytest.approx(0.01)
    # an empty comparison reports zero, an all-zero reference does not divide by zero
    assert error_report(np.zeros(0), np.zeros(0), np.ones(3))["E"] == 0.0
    assert error_report(np.array([0.5]), np.array([0.0]), np.array([0.0]))["E"] == pytest.approx(0.5)


def test_structured_points_cover_the_tile_boundaries():
    from oracle.compare import sample_points, structured_points
    n, c_out, h, w, band, strip = 3, 130, 10, 50, 4, 16
    rpi = h + 1
    pts = structured_points(n, c_out, h, w, band, strip, rpi, seed=1)
    assert pts.dtype == np.int32 and pts.shape[1] == 4
    assert (pts >= 0).all() and (pts[:, 0] < n).all() and (pts[:, 1] < c_out).all() and (pts[:, 2] < h).all() and (pts[:, 3] < w).all()
    cells = {(int(a), int(c), int(d)) for a, _, c, d in pts}
    vrows = n * rpi - 1
    for k in range(1, (vrows + band - 1) // band):              # both sides of every band boundary that is an image row
        for v in (k * band - 1, k * band):
            if v % rpi < h:
                assert any(img == v // rpi and oy == v % rpi for img, oy, _ in cells), v
    for k in range(1, (w + strip - 1) // strip):                # both sides of every strip boundary
        for x in (k * strip - 1, k * strip):
            assert any(ox == x for _, _, ox in cells), x
    for img in range(n):                                         # first and last row of every image
        assert any(i == img and oy == 0 for i, oy, _ in cells) and any(i == img and oy == h - 1 for i, oy, _ in cells)
    last_v0, last_x0 = ((vrows - 1) // band) * band, ((w - 1) // strip) * strip
    for v in range(last_v0, vrows):                              # the whole last tile
        for x in range(last_x0, w):
            if v % rpi < h:
                assert (v // rpi, v % rpi, x) in cells
    assert set(int(f) for f in pts[:, 1]) <= {0, 63, 64, 127, 128, 129}
    rnd = sample_points(n, c_out, h, w, 100, seed=2)
    assert rnd.shape == (100 + 36, 4) and (rnd[:, 1] < c_out).all()
