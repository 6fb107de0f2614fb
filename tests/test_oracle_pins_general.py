"""Pins for the CPU checker's other kernel sizes, strides and pooled results: each test ties
oracle/ to something other than itself (a hand-worked example, an identity with the pinned 3x3
stride-1 definition, a library routine, a brute-force gather)."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny(seed, ksize, taps, stride, n=2, c_in=3, c_out=4, h=7, w=6, keep=0.6, npat=5):
    pset = synth.random_pattern_set(ksize, taps, min(npat, 1 if ksize == 1 else npat), seed)
    lay = synth.random_pruned_layer_k("tiny", n, c_in, c_out, h, w, "f32", ksize, pset, keep, 0.5, seed, stride=stride)
    return lay, lay.make_input().astype(np.float64)


def numpy_dense_weights(lay):
    """Independent construction of the masked dense weights from the mask bits."""
    k = lay.ksize
    wd = np.zeros((lay.c_out, lay.c_in, k, k))
    for kid in range(lay.c_out * lay.c_in):
        if not lay.conn_mask[kid]:
            continue
        co, ci = divmod(kid, lay.c_in)
        taps = [t for t in range(k * k) if (int(lay.pattern_masks[lay.pattern_id[kid]]) >> t) & 1]
        for j, t in enumerate(taps):
            wd[co, ci, t // k, t % k] = lay.weights[kid, j]
    return wd


@pytest.mark.parametrize("case", ["stride2_3x3", "stride1_5x5", "conn_1x1"])
def test_hand_worked_examples(case):
    g = json.load(open(os.path.join(GOLDEN, "hand_conv_general.json")))[case]
    w = np.array(g["weights"], dtype=np.float64)
    taps = w.shape[1]
    wd = oracle.expand_weights_k(g["c_in"], g["c_out"], g["ksize"], g["pattern_masks"], g["pattern_id"], g["conn_mask"], w, taps)
    x = np.array(g["x"], dtype=np.float64)[None]
    want = np.array(g["y"], dtype=np.float64)
    y = oracle.conv_k(x, wd, g["stride"], np.array(g["bias"]))
    assert np.array_equal(y[0], want)
    yb = oracle.brute_k(x, g["ksize"], g["stride"], taps, g["pattern_masks"], g["pattern_id"], g["conn_mask"], w,
                        g["c_out"], np.array(g["bias"]))
    assert np.array_equal(yb[0], want)
    pts = np.array([[0, co, oy, ox] for co in range(want.shape[0]) for oy in range(want.shape[1])
                    for ox in range(want.shape[2])], dtype=np.int32)
    ya, _, _ = oracle.conv_k_at(x.astype(np.float32), wd, pts, g["stride"], np.array(g["bias"]))
    assert np.array_equal(ya.reshape(want.shape), want)


@pytest.mark.parametrize("ksize,taps", [(1, 1), (3, 4), (5, 4), (5, 9), (7, 6)])
@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("shape", [(7, 6), (1, 1), (1, 8), (5, 1), (8, 9)])
def test_expand_brute_and_library_convolution(ksize, taps, stride, shape):
    h, w = shape
    for seed in (0, 1):
        lay, x = tiny(seed, ksize, taps, stride, h=h, w=w)
        wd = oracle.layer_dense_weights(lay)
        assert np.array_equal(wd, numpy_dense_weights(lay))
        for relu in (False, True):
            y = oracle.conv_k(x, wd, stride, lay.bias, relu)
            yb = oracle.brute_k(x, ksize, stride, taps, lay.pattern_masks, lay.pattern_id, lay.conn_mask,
                                lay.weights.astype(np.float64), lay.c_out, lay.bias, relu)
            assert y.shape == (lay.n, lay.c_out, lay.conv_h, lay.conv_w) == yb.shape
            assert np.allclose(y, yb, rtol=0, atol=1e-13)
            t = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(numpy_dense_weights(lay)),
                                           torch.from_numpy(lay.bias.astype(np.float64)), stride=stride, padding=ksize // 2)
            if relu:
                t = torch.relu(t)
            assert np.allclose(y, t.numpy(), rtol=0, atol=1e-12)


def test_3x3_stride_1_is_the_pinned_definition_and_stride_2_is_every_second_output():
    for seed in (0, 1, 2):
        lay = synth.random_pruned_layer("t", 2, 5, 6, 9, 8, "f32", synth.PSET16, 0.5, 0.5, seed)
        x = lay.make_input().astype(np.float64)
        wd = oracle.layer_dense_weights(lay)
        y1, pre1, sc1 = oracle.conv(x, wd, lay.bias, True, want_pre=True, want_scale=True)
        yk, prek, sck = oracle.conv_k(x, wd, 1, lay.bias, True, want_pre=True, want_scale=True)
        assert np.array_equal(y1, yk) and np.array_equal(pre1, prek) and np.array_equal(sc1, sck)
        y2, pre2, sc2 = oracle.conv_k(x, wd, 2, lay.bias, True, want_pre=True, want_scale=True)
        assert np.array_equal(y2, y1[:, :, ::2, ::2]) and np.array_equal(pre2, pre1[:, :, ::2, ::2])
        assert np.array_equal(sc2, sc1[:, :, ::2, ::2])


def test_1x1_is_a_matrix_product():
    lay, x = tiny(3, 1, 1, 1, n=2, c_in=7, c_out=5, h=4, w=6)
    wd = oracle.layer_dense_weights(lay)
    wm = np.where(lay.conn_mask.reshape(5, 7) != 0, lay.weights.reshape(5, 7).astype(np.float64), 0.0)
    assert np.array_equal(wd[:, :, 0, 0], wm)
    y = oracle.conv_k(x, wd, 1, None, False)
    want = np.einsum("oc,nchw->nohw", wm, x)
    assert np.allclose(y, want, rtol=0, atol=1e-13)


def test_sampled_evaluation_equals_full_evaluation():
    for ksize, taps, stride in [(5, 6, 2), (3, 4, 2), (1, 1, 1), (7, 5, 1)]:
        lay, x = tiny(4, ksize, taps, stride, h=9, w=11)
        wd = oracle.layer_dense_weights(lay)
        y, pre, sc = oracle.conv_k(x, wd, stride, lay.bias, True, want_pre=True, want_scale=True)
        rs = np.random.RandomState(0)
        pts = np.stack([rs.randint(0, lay.n, 200), rs.randint(0, lay.c_out, 200), rs.randint(0, lay.conv_h, 200),
                        rs.randint(0, lay.conv_w, 200)], axis=1).astype(np.int32)
        for xs in (x.astype(np.float32), x.astype(np.float16)):
            yf, pf, sf = oracle.conv_k(xs.astype(np.float64), wd, stride, lay.bias, True, want_pre=True, want_scale=True)
            ya, pa, sa = oracle.conv_k_at(np.ascontiguousarray(xs), wd, pts, stride, lay.bias, True)
            idx = (pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3])
            assert np.array_equal(ya, yf[idx]) and np.array_equal(pa, pf[idx]) and np.array_equal(sa, sf[idx])


def test_layer_reference_with_a_fused_pool_is_the_library_pool_of_the_activated_result():
    pset = synth.random_pattern_set(3, 4, 6, 0)
    lay = synth.random_pruned_layer_k("p", 2, 4, 5, 8, 10, "f32", 3, pset, 0.5, 0.5, 0, pool=True)
    x = lay.make_input().astype(np.float64)
    y, pre, sc = oracle.layer_reference(lay, x)
    assert y.shape == (2, 5, 4, 5) and pre.shape == (2, 5, 8, 10)
    t = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(numpy_dense_weights(lay)),
                                   torch.from_numpy(lay.bias.astype(np.float64)), padding=1)
    t = torch.nn.functional.max_pool2d(torch.relu(t), 2)
    assert np.allclose(y, t.numpy(), rtol=0, atol=1e-12)


def test_invalid_descriptions_are_rejected():
    with pytest.raises(ValueError):
        oracle.expand_weights_k(1, 1, 4, [1], [0], [1], np.ones(1), 1)            # even kernel size
    with pytest.raises(ValueError):
        oracle.expand_weights_k(1, 1, 3, [1 << 9], [0], [1], np.ones(1), 1)       # bit outside the window
    with pytest.raises(ValueError):
        oracle.expand_weights_k(1, 1, 3, [3], [0], [1], np.ones(1), 1)            # two bits, one tap declared
    with pytest.raises(ValueError):
        oracle.expand_weights_k(1, 1, 3, [1], [1], [1], np.ones(1), 1)            # pattern id out of range
