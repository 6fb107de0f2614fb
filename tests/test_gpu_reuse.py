"""GPU parity of deep reuse (paper, section 2.3.2) against the CPU checker, through the C ABI: signatures and
representatives bit-exact (integer decisions, taken in binary32 in the same order on both sides), outputs within
the fp32 tolerance."""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle.compare import TOL, error_report
import paper_2206_10620_amd as pp

pytestmark = pytest.mark.gpu


def check(lay, n=None, n_max=None):
    x = lay.make_input(n)
    n = x.shape[0]
    print(f"case {lay.name} n={n} k={lay.k} m={lay.m} L={lay.seg_len} H={lay.hash_bits}", flush=True)
    plan = pp.reuse_plan_from_layer(lay, n_max=n_max if n_max is not None else n)
    try:
        xd = torch.from_numpy(x).cuda()
        yd = torch.full((n, lay.m), float("nan"), dtype=torch.float32, device="cuda")
        plan.run(xd, yd)
        torch.cuda.synchronize()
        sig, rep = plan.clusters(n)
        got = yd.cpu().numpy()
    finally:
        plan.close()
    ref, pre, sc, rsig, rrep = oracle.reuse_layer(x, lay.weights, lay.hyperplanes, lay.seg_len, lay.hash_bits, lay.bias, lay.relu)
    assert np.array_equal(sig, rsig), "signatures differ"
    assert np.array_equal(rep, rrep), "representatives differ"
    assert not np.isnan(got).any()
    r = error_report(got, ref, pre, sc)
    assert r["E"] <= TOL["f32"], r
    return rep


# n, k, m, L, H
SHAPES = [
    (1, 8, 1, 8, 1),
    (7, 12, 5, 3, 2),
    (256, 32, 16, 8, 4),
    (257, 32, 16, 8, 4),            # one row into a second workgroup
    (1000, 96, 33, 32, 12),         # longest neuron vector, most hash bits, odd output count
    (3000, 60, 64, 5, 7),
    (5000, 576, 64, 16, 8),         # the benchmark's segmenting
    (700, 16, 8, 1, 3),             # neuron vectors of one value
]


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(str(v) for v in s))
def test_small_shapes(shape, relu):
    n, k, m, L, H = shape
    lay = synth.random_reuse_layer("r", n, k, m, L, H, seed=n + k, relu=relu, prototypes=16, noise=0.02)
    check(lay)


def test_values_on_the_hash_boundary_and_no_bias():
    # integer inputs and hyperplanes give many projections that are exactly zero: "> 0" must read them as 0 on both sides
    lay = synth.random_reuse_layer("z", 600, 24, 6, 6, 5, seed=3, with_bias=False)
    rs = np.random.RandomState(0)
    lay.hyperplanes = rs.randint(-2, 3, lay.hyperplanes.shape).astype(np.float32)
    lay.make_input = lambda n=None: rs.randint(-3, 4, (600, 24)).astype(np.float32)
    check(lay)


def test_fewer_rows_than_the_plan_was_sized_for_and_a_second_run():
    lay = synth.random_reuse_layer("p", 2000, 64, 32, 16, 6, seed=5)
    check(lay, n=300, n_max=2000)
    plan = pp.reuse_plan_from_layer(lay)
    try:
        xa, xb = torch.from_numpy(lay.make_input()).cuda(), torch.from_numpy(lay.make_input(500)).cuda()
        ya = plan.run(xa)
        yb = plan.run(xb)                       # representatives of the first run must not leak into the second
        torch.cuda.synchronize()
        sig, rep = plan.clusters(500)
    finally:
        plan.close()
    ref, pre, sc, rsig, rrep = oracle.reuse_layer(lay.make_input(500), lay.weights, lay.hyperplanes, lay.seg_len, lay.hash_bits, lay.bias, lay.relu)
    assert np.array_equal(sig, rsig) and np.array_equal(rep, rrep)
    assert error_report(yb.cpu().numpy(), ref, pre, sc)["E"] <= TOL["f32"]


def test_identical_vectors_give_the_exact_product():
    lay = synth.random_reuse_layer("x", 4000, 64, 16, 8, 12, seed=10, prototypes=6, noise=0.0, relu=False)
    rep = check(lay)
    x = lay.make_input()
    assert (rep >= 0).sum() == 6 * lay.segments          # no two prototypes share a signature with this seed
    plan = pp.reuse_plan_from_layer(lay)
    try:
        y = plan.run(torch.from_numpy(x).cuda()).cpu().numpy()
    finally:
        plan.close()
    exact = x.astype(np.float64) @ lay.weights.astype(np.float64) + lay.bias.astype(np.float64)
    assert np.abs(y - exact).max() <= 1e-5 * max(1.0, np.abs(exact).max())


def test_benchmark_layer_full_size():
    lay = synth.conv_shaped_reuse_layer()
    rep = check(lay)
    print("clusters used", int((rep >= 0).sum()), "of", lay.n * lay.segments, "neuron vectors", flush=True)


def test_the_comparison_fails_on_a_wrong_layer():
    """Negative controls.  The GPU runs the layer as given; the checker is handed a copy with one mistake planted
    in it on the CPU side: one hyperplane negated (signatures must differ), the election of the highest row instead
    of the lowest (representatives must differ), one weight off by 25 x the tolerance (E must exceed it)."""
    lay = synth.random_reuse_layer("neg", 1500, 64, 16, 8, 6, seed=9, prototypes=12, noise=0.05)
    x = lay.make_input()
    plan = pp.reuse_plan_from_layer(lay)
    try:
        got = plan.run(torch.from_numpy(x).cuda()).cpu().numpy()
        torch.cuda.synchronize()
        sig, rep = plan.clusters(lay.n)
    finally:
        plan.close()
    ref, pre, sc, rsig, rrep = oracle.reuse_layer(x, lay.weights, lay.hyperplanes, lay.seg_len, lay.hash_bits, lay.bias, lay.relu)
    assert np.array_equal(sig, rsig) and np.array_equal(rep, rrep) and error_report(got, ref, pre, sc)["E"] <= TOL["f32"]
    hp = lay.hyperplanes.copy()
    hp.reshape(-1, lay.seg_len)[3] *= -1.0
    assert not np.array_equal(sig, oracle.reuse_signatures(x, hp, lay.seg_len, lay.hash_bits))
    # the last row of every cluster instead of the first: the checker's election run on the rows in reverse
    last = oracle.reuse_representatives(np.ascontiguousarray(rsig[::-1]), lay.hash_bits)
    last = np.where(last >= 0, lay.n - 1 - last, -1)
    assert not np.array_equal(rep, last)
    w = lay.weights.copy()
    r, c = np.unravel_index(int(np.argmax(np.abs(w))), w.shape)
    w[r, c] *= 1.0 + 25 * TOL["f32"]
    wref, wpre, wsc, _, _ = oracle.reuse_layer(x, w, lay.hyperplanes, lay.seg_len, lay.hash_bits, lay.bias, lay.relu)
    assert error_report(got, wref, wpre, wsc)["E"] > TOL["f32"]
