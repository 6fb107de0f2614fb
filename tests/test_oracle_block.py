"""Pins for the CPU checker of the block-pruned matrix product (paper, section 2.1.2).

Each test fixes the checker to something other than itself: a hand-worked fixture, numpy's float64
matrix product on a mask built another way, a gather-style evaluation that never forms the masked
matrix, closed forms and invariants.
"""
import json
import os

import numpy as np
import pytest

import oracle
import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_block_gemm.json")


def small_layers():
    return [
        synth.random_block_layer("a", 8, 8, 5, 4, 4, "f32", 0.6, 0.6, 1),
        synth.random_block_layer("ragged_blocks", 10, 13, 7, 4, 5, "f32", 0.5, 0.7, 2),
        synth.random_block_layer("one_block", 6, 9, 3, 6, 9, "f32", 0.5, 0.5, 3),
        synth.random_block_layer("unit_blocks", 5, 6, 4, 1, 1, "f32", 0.5, 0.9, 4),
        synth.random_block_layer("wide", 3, 40, 2, 2, 16, "f32", 0.8, 0.3, 5, relu=True),
        synth.random_block_layer("tall", 33, 4, 6, 8, 2, "f32", 0.4, 0.8, 6, relu=True, with_bias=False),
    ]


def test_hand_fixture():
    g = json.load(open(GOLD))
    wd = oracle.block_expand(g["m"], g["k"], g["bm"], g["bk"], np.array(g["row_keep"]), np.array(g["col_keep"]),
                             np.array(g["weights"], dtype=np.float64))
    assert np.array_equal(wd, np.array(g["wd"], dtype=np.float64))
    x = np.array(g["x"], dtype=np.float64)
    y, pre = oracle.gemm(wd, x, np.array(g["bias"]), relu=True, want_pre=True)
    assert np.array_equal(pre, np.array(g["pre"]))
    assert np.array_equal(y, np.array(g["y_relu"]))
    assert np.array_equal(oracle.gemm(wd, x, np.array(g["bias"]), relu=False), np.array(g["pre"]))
    yb = oracle.block_brute(g["m"], g["k"], g["bm"], g["bk"], np.array(g["row_keep"]), np.array(g["col_keep"]),
                            np.array(g["weights"], dtype=np.float64), x, np.array(g["bias"]), relu=True)
    assert np.array_equal(yb, np.array(g["y_relu"]))


@pytest.mark.parametrize("lay", small_layers(), ids=lambda l: l.name)
def test_against_numpy_product_on_a_mask_built_by_broadcasting(lay):
    wd = oracle.block_expand(lay.m, lay.k, lay.bm, lay.bk, lay.row_keep, lay.col_keep, lay.weights)
    keep = lay.keep_matrix()
    assert np.array_equal(wd != 0, keep & (lay.weights != 0))
    assert np.array_equal(wd, np.where(keep, lay.weights.astype(np.float64), 0.0))
    x = lay.make_input().astype(np.float64)
    y, pre, sc = oracle.gemm(wd, x, lay.bias, lay.relu, want_pre=True, want_scale=True)
    b = 0.0 if lay.bias is None else lay.bias.astype(np.float64)[:, None]
    ref = np.where(keep, lay.weights.astype(np.float64), 0.0) @ x + b
    assert np.allclose(pre, ref, rtol=0, atol=1e-12 * max(1.0, np.abs(ref).max()))
    assert np.allclose(y, np.maximum(ref, 0) if lay.relu else ref, rtol=0, atol=1e-12 * max(1.0, np.abs(ref).max()))
    ref_sc = np.abs(np.where(keep, lay.weights.astype(np.float64), 0.0)) @ np.abs(x) + np.abs(b)
    assert np.allclose(sc, ref_sc, rtol=1e-12)


@pytest.mark.parametrize("lay", small_layers(), ids=lambda l: l.name)
def test_against_the_gather_evaluation(lay):
    x = lay.make_input().astype(np.float64)
    y, _, _ = oracle.block_layer_reference(lay, x)
    yb = oracle.block_brute(lay.m, lay.k, lay.bm, lay.bk, lay.row_keep, lay.col_keep, lay.weights, x, lay.bias, lay.relu)
    assert np.allclose(y, yb, rtol=0, atol=1e-12 * max(1.0, np.abs(yb).max()))


def test_pruned_positions_never_matter():
    lay = synth.random_block_layer("p", 12, 12, 4, 4, 3, "f32", 0.5, 0.5, 7, poison=True)
    x = lay.make_input().astype(np.float64)
    y0, _, _ = oracle.block_layer_reference(lay, x)
    keep = lay.keep_matrix()
    assert (~keep).any() and np.all(lay.weights[~keep] == 1000.0)
    lay.weights = np.where(keep, lay.weights, np.float32(-7.0))
    y1, _, _ = oracle.block_layer_reference(lay, x)
    assert np.array_equal(y0, y1)


def test_all_kept_is_the_dense_product_and_nothing_kept_is_the_bias():
    m, k, n, bm, bk = 7, 9, 5, 3, 4
    rng = np.random.default_rng(0)
    w, x, b = rng.standard_normal((m, k)), rng.standard_normal((k, n)), rng.standard_normal(m)
    nb = ((m + bm - 1) // bm) * ((k + bk - 1) // bk)
    ones_r, ones_c = np.ones(nb * bm, np.uint8), np.ones(nb * bk, np.uint8)
    wd = oracle.block_expand(m, k, bm, bk, ones_r, ones_c, w)
    assert np.array_equal(wd, w)
    assert np.allclose(oracle.gemm(wd, x, b), w @ x + b[:, None], atol=1e-13)
    for rk, ck in ((0 * ones_r, ones_c), (ones_r, 0 * ones_c)):
        wd0 = oracle.block_expand(m, k, bm, bk, rk, ck, w)
        assert not wd0.any()
        assert np.array_equal(oracle.gemm(wd0, x, b), np.repeat(b[:, None], n, axis=1))
        assert np.array_equal(oracle.gemm(wd0, x, b, relu=True), np.repeat(np.maximum(b, 0)[:, None], n, axis=1))


def test_one_kept_element_gives_a_scaled_row_of_x():
    m, k, n, bm, bk = 6, 8, 4, 2, 4
    blocks_k = 2
    w = np.arange(1, m * k + 1, dtype=np.float64).reshape(m, k)
    x = np.random.default_rng(1).standard_normal((k, n))
    for (r, c) in ((0, 0), (3, 5), (5, 7), (2, 3)):
        rk = np.zeros((3, blocks_k, bm), np.uint8)
        ck = np.zeros((3, blocks_k, bk), np.uint8)
        rk[r // bm, c // bk, r % bm] = 1
        ck[r // bm, c // bk, c % bk] = 1
        y = oracle.gemm(oracle.block_expand(m, k, bm, bk, rk, ck, w), x)
        want = np.zeros((m, n))
        want[r] = w[r, c] * x[c]
        assert np.array_equal(y, want)


def test_row_flags_and_column_flags_are_not_interchanged():
    # a block that keeps one row and all columns yields a full row of that block; the transposed reading would give a column
    m = k = 4
    w = np.arange(1, 17, dtype=np.float64).reshape(4, 4)
    rk = np.zeros((1, 1, 4), np.uint8)
    ck = np.ones((1, 1, 4), np.uint8)
    rk[0, 0, 2] = 1
    wd = oracle.block_expand(m, k, 4, 4, rk, ck, w)
    want = np.zeros((4, 4))
    want[2] = w[2]
    assert np.array_equal(wd, want)


def test_linearity_in_x_without_the_activation():
    lay = synth.random_block_layer("lin", 9, 14, 6, 3, 7, "f32", 0.6, 0.6, 11, with_bias=False)
    x1 = lay.make_input().astype(np.float64)
    x2 = np.random.default_rng(2).standard_normal(x1.shape)
    f = lambda x: oracle.block_layer_reference(lay, x, relu=False)[0]
    assert np.allclose(f(2.0 * x1 - 3.0 * x2), 2.0 * f(x1) - 3.0 * f(x2), atol=1e-12)


def test_sampled_evaluation_equals_the_full_one():
    lay = synth.random_block_layer("pts", 20, 24, 9, 4, 8, "f16", 0.6, 0.6, 12, relu=True)
    x = lay.make_input().astype(np.float64)
    y, pre, sc = oracle.block_layer_reference(lay, x)
    w = oracle.widen_f16(oracle.round_f16(lay.weights.astype(np.float64)))
    wd = oracle.block_expand(lay.m, lay.k, lay.bm, lay.bk, lay.row_keep, lay.col_keep, w)
    pts = np.array([(r, j) for r in (0, 3, 19) for j in (0, 4, 8)], dtype=np.int32)
    ya, prea, sca = oracle.gemm_at(wd, x, pts, lay.bias, True)
    assert np.array_equal(ya, y[pts[:, 0], pts[:, 1]])
    assert np.array_equal(prea, pre[pts[:, 0], pts[:, 1]])
    assert np.array_equal(sca, sc[pts[:, 0], pts[:, 1]])


def test_f16_layers_use_rounded_weights():
    lay = synth.random_block_layer("h", 8, 8, 3, 4, 4, "f16", 0.7, 0.7, 13, poison=False)
    x = lay.make_input()
    assert x.dtype == np.float16
    y, _, _ = oracle.block_layer_reference(lay, x.astype(np.float64), relu=False)
    w16 = np.where(lay.keep_matrix(), lay.weights.astype(np.float16).astype(np.float64), 0.0)
    ref = w16 @ x.astype(np.float64) + lay.bias.astype(np.float64)[:, None]
    assert np.allclose(y, ref, atol=1e-12)
