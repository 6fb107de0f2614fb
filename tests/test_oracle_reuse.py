"""Pins for the CPU checker of deep reuse (paper, section 2.3.2)."""
import json
import os

import numpy as np

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_deep_reuse.json")


def numpy_substitution(x, w, sig, bias, relu):
    """The approximation written a second way: replace every neuron vector by the first row of X that has the
    same signature in that segment (numpy's first-occurrence search), then take the exact product."""
    n, k = x.shape
    S = sig.shape[1]
    L = k // S
    xs = np.empty_like(x, dtype=np.float64)
    for s in range(S):
        _, first, inverse = np.unique(sig[:, s], return_index=True, return_inverse=True)
        xs[:, s * L:(s + 1) * L] = x[first[inverse.ravel()], s * L:(s + 1) * L]
    pre = xs @ w.astype(np.float64) + (0.0 if bias is None else np.asarray(bias, dtype=np.float64)[None, :])
    return np.maximum(pre, 0.0) if relu else pre


def test_hand_fixture():
    g = json.load(open(GOLD))
    x, w, hp = np.array(g["x"], np.float32), np.array(g["w"], np.float32), np.array(g["hyperplanes"], np.float32)
    y, pre, sc, sig, rep = oracle.reuse_layer(x, w, hp, g["seg_len"], g["hash_bits"], np.array(g["bias"]), relu=True)
    assert np.array_equal(sig, np.array(g["signatures"]))
    assert np.array_equal(rep, np.array(g["representatives"]))
    assert np.array_equal(pre, np.array(g["pre"]))
    assert np.array_equal(y, np.array(g["y_relu"]))
    y2 = oracle.reuse_layer(x, w, hp, g["seg_len"], g["hash_bits"], np.array(g["bias"]), relu=False)[0]
    assert np.array_equal(y2, np.array(g["pre"]))


def test_signatures_against_numpy_on_integer_inputs():
    # integer-valued inputs: every binary32 partial sum is exact, so any summation order gives the same sign
    rs = np.random.RandomState(0)
    n, k, L, H = 200, 24, 6, 5
    x = rs.randint(-8, 9, (n, k)).astype(np.float32)
    hp = rs.randint(-3, 4, (k // L, H, L)).astype(np.float32)
    sig = oracle.reuse_signatures(x, hp, L, H)
    proj = np.einsum("nsl,shl->nsh", x.reshape(n, k // L, L).astype(np.int64), hp.astype(np.int64))
    want = ((proj > 0).astype(np.int64) << np.arange(H)[None, None, :]).sum(axis=2)
    assert np.array_equal(sig, want.astype(np.uint16))
    assert (proj == 0).any()                      # the "> 0" boundary is exercised
    rep = oracle.reuse_representatives(sig, H)
    for s in range(k // L):
        for gg in range(1 << H):
            rows = np.nonzero(sig[:, s] == gg)[0]
            assert rep[s, gg] == (rows[0] if len(rows) else -1)


def test_identical_vectors_inside_every_cluster_give_the_exact_product():
    # x in {-1, +1} and axis-aligned hyperplanes (H = L): the signature IS the vector, so clusters hold identical vectors
    rs = np.random.RandomState(1)
    n, k, L, m = 300, 12, 4, 7
    x = (rs.randint(0, 2, (n, k)) * 2 - 1).astype(np.float32)
    hp = np.tile(np.eye(L, dtype=np.float32)[None], (k // L, 1, 1))
    w = rs.standard_normal((k, m)).astype(np.float32)
    b = rs.standard_normal(m).astype(np.float32)
    y, pre, sc, sig, rep = oracle.reuse_layer(x, w, hp, L, L, b, relu=False)
    exact = x.astype(np.float64) @ w.astype(np.float64) + b.astype(np.float64)
    assert np.allclose(y, exact, rtol=0, atol=1e-12)
    assert (rep >= 0).sum() < n * (k // L) / 4                  # and it did reuse: far fewer clusters than vectors
    assert np.allclose(sc, np.abs(x).astype(np.float64) @ np.abs(w).astype(np.float64) + np.abs(b), atol=1e-12)


def test_zero_hyperplanes_give_every_row_the_result_of_row_zero():
    rs = np.random.RandomState(2)
    n, k, L, H, m = 9, 8, 4, 3, 5
    x, w = rs.standard_normal((n, k)).astype(np.float32), rs.standard_normal((k, m)).astype(np.float32)
    y, _, _, sig, rep = oracle.reuse_layer(x, w, np.zeros((k // L, H, L), np.float32), L, H)
    assert not sig.any() and np.all(rep[:, 0] == 0) and np.all(rep[:, 1:] == -1)
    row0 = x[0].astype(np.float64) @ w.astype(np.float64)
    assert np.allclose(y, np.tile(row0, (n, 1)), atol=1e-12)


def test_equals_the_exact_product_of_the_substituted_input():
    rs = np.random.RandomState(3)
    n, k, L, H, m = 500, 32, 8, 12, 6
    # rows that resemble each other (the redundancy the method lives on): a few prototypes plus small noise
    x = (rs.standard_normal((12, k))[rs.randint(0, 12, n)] + 0.01 * rs.standard_normal((n, k))).astype(np.float32)
    hp = rs.standard_normal((k // L, H, L)).astype(np.float32)
    w = rs.standard_normal((k, m)).astype(np.float32)
    b = rs.standard_normal(m).astype(np.float32)
    for relu in (False, True):
        y, pre, sc, sig, rep = oracle.reuse_layer(x, w, hp, L, H, b, relu)
        want = numpy_substitution(x.astype(np.float64), w, sig, b, relu)
        assert np.allclose(y, want, rtol=0, atol=1e-11)
    # an approximation: it differs from the exact product, by about the noise between similar vectors
    exact = x.astype(np.float64) @ w.astype(np.float64) + b
    err = np.linalg.norm(pre - exact) / np.linalg.norm(exact)
    assert 1e-5 < err < 0.5, err
    assert (rep >= 0).sum() < 0.5 * n * (k // L)


def test_permuting_output_columns_permutes_the_result():
    rs = np.random.RandomState(4)
    n, k, L, H, m = 40, 12, 3, 3, 5
    x, w = rs.standard_normal((n, k)).astype(np.float32), rs.standard_normal((k, m)).astype(np.float32)
    hp = rs.standard_normal((k // L, H, L)).astype(np.float32)
    perm = rs.permutation(m)
    y = oracle.reuse_layer(x, w, hp, L, H)[0]
    yp = oracle.reuse_layer(x, w[:, perm], hp, L, H)[0]
    assert np.array_equal(yp, y[:, perm])
