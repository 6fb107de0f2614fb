"""GPU parity: the HIP library (through its C ABI) against the CPU checker on the same seeded inputs.

Tolerances (max over outputs of |gpu - ref| / max(|ref|, rms of the reference pre-activations)):
1e-5 for fp32 storage, 2e-3 for fp16 storage with fp32 accumulation.  Plan metadata is compared
bit-exactly in the host tests."""
import copy
import sys

import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2206_10620_amd as pp
from gpu_util import check_layer, run_layer, to_device

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def T(**kw):
    return pp.Tuning(**kw)


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("relu", [True, False])
def test_config1_small_layer(seed, relu):
    lay = synth.config1(seed)
    say(f"config1 seed={seed} relu={relu}")
    rep, _ = check_layer(lay, relu=relu, label="cfg1")
    say(f"  E={rep['E']:.2e} {rep['chosen']}")


@pytest.mark.parametrize("relu", [True, False])
def test_config1_generic_kernel(relu):
    lay = synth.config1(0)
    rep, _ = check_layer(lay, tuning=T(variant=1), relu=relu, label="cfg1-generic")
    assert rep["chosen"]["variant"] == 1


# (n, c_in, c_out, h, w): ragged widths, single rows/columns, channel counts that are not multiples of
# the chunk, filter counts that are not multiples of the filters per wave, several images per tile.
SHAPES = [(1, 3, 5, 1, 1), (2, 5, 9, 1, 7), (3, 4, 4, 9, 1), (2, 7, 13, 7, 7), (3, 9, 10, 14, 14), (1, 6, 6, 5, 30),
          (2, 10, 17, 11, 33), (1, 19, 8, 28, 28), (5, 8, 24, 3, 56), (1, 12, 8, 20, 130), (2, 33, 40, 6, 64)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_ragged_shapes(shape, dtype):
    n, c_in, c_out, h, w = shape
    say(f"ragged {shape} {dtype}")
    lay = synth.random_pruned_layer("ragged", n, c_in, c_out, h, w, dtype, synth.PSET16, 0.6, 0.3, seed=n + w)
    for relu in (True, False):
        rep, _ = check_layer(lay, tuning=T(variant=2), relu=relu, label=f"ragged{shape}")
    say(f"  E={rep['E']:.2e} {rep['chosen']}")


TUNINGS = [dict(filters_per_wave=4, rows_per_lane=1, lanes_x=2), dict(filters_per_wave=8, rows_per_lane=2, lanes_x=4),
           dict(filters_per_wave=16, rows_per_lane=1, lanes_x=7), dict(filters_per_wave=8, rows_per_lane=2, lanes_x=8),
           dict(filters_per_wave=4, rows_per_lane=2, lanes_x=14), dict(filters_per_wave=8, rows_per_lane=1, lanes_x=16),
           dict(filters_per_wave=8, rows_per_lane=2, lanes_x=16, waves_f=2, split_c=4, chunk_c=8),
           dict(filters_per_wave=4, rows_per_lane=1, lanes_x=8, waves_f=1, split_c=8, chunk_c=16),
           dict(filters_per_wave=8, rows_per_lane=2, lanes_x=7, waves_f=3, split_c=2, chunk_c=6),
           dict(filters_per_wave=8, rows_per_lane=1, lanes_x=14, waves_f=16, split_c=1, chunk_c=1),
           dict(filters_per_wave=4, rows_per_lane=4, lanes_x=16, waves_f=4, split_c=2, chunk_c=4),
           dict(filters_per_wave=4, rows_per_lane=4, lanes_x=7, waves_f=2, split_c=1, chunk_c=5),
           dict(filters_per_wave=4, rows_per_lane=2, lanes_x=14, waves_f=4, split_c=2, chunk_c=8, balance=1),
           dict(filters_per_wave=4, rows_per_lane=2, lanes_x=14, waves_f=4, split_c=2, chunk_c=8, balance=2),
           dict(filters_per_wave=4, rows_per_lane=1, lanes_x=16, waves_f=8, split_c=1, chunk_c=8),
           dict(filters_per_wave=4, rows_per_lane=2, lanes_x=8, waves_f=2, split_c=4, chunk_c=8)]


@pytest.mark.parametrize("tune", TUNINGS)
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_every_tile_geometry(tune, dtype):
    say(f"tuning {tune} {dtype}")
    for (n, c_in, c_out, h, w) in [(2, 21, 37, 19, 45), (3, 16, 16, 8, 8), (2, 9, 12, 11, 48)]:
        lay = synth.random_pruned_layer("tune", n, c_in, c_out, h, w, dtype, synth.PSET16, 0.5, 0.3, seed=7)
        rep, _ = check_layer(lay, tuning=T(variant=2, **tune), label=f"tune{tune}")
        for k, v in tune.items():
            assert rep["chosen"][k] == v
    say(f"  E={rep['E']:.2e}")


# How input tiles reach LDS: 1 = through registers, k >= 2 = direct loads into a ring of k buffers.
# Shapes: rows on 16-byte boundaries (16-byte slots), on 4-byte boundaries only (4-byte slots), and
# c_in / chunk_c combinations with fewer chunks than buffers, exactly as many, and many more; a
# one-wavefront workgroup (more load instructions per channel than wavefronts) and a 16-wavefront one.
STAGINGS = [(1, dict(filters_per_wave=4, rows_per_lane=2, lanes_x=8, waves_f=4, split_c=2, chunk_c=4)),
            (2, dict(filters_per_wave=4, rows_per_lane=2, lanes_x=8, waves_f=4, split_c=2, chunk_c=4)),
            (1, dict(filters_per_wave=4, rows_per_lane=2, lanes_x=8, waves_f=4, split_c=2, chunk_c=4, balance=1)),
            (2, dict(filters_per_wave=4, rows_per_lane=2, lanes_x=8, waves_f=4, split_c=2, chunk_c=4, balance=1)),
            (3, dict(filters_per_wave=4, rows_per_lane=1, lanes_x=14, waves_f=1, split_c=1, chunk_c=3)),
            (4, dict(filters_per_wave=8, rows_per_lane=2, lanes_x=16, waves_f=8, split_c=2, chunk_c=2)),
            (8, dict(filters_per_wave=4, rows_per_lane=4, lanes_x=4, waves_f=2, split_c=1, chunk_c=1)),
            (3, dict(filters_per_wave=16, rows_per_lane=1, lanes_x=7, waves_f=2, split_c=1, chunk_c=5)),
            (5, dict(filters_per_wave=4, rows_per_lane=2, lanes_x=2, waves_f=16, split_c=1, chunk_c=7))]


@pytest.mark.parametrize("staging,tune", STAGINGS)
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_staging_paths(staging, tune, dtype):
    say(f"staging {staging} {tune} {dtype}")
    for (n, c_in, c_out, h, w) in [(2, 23, 40, 19, 48), (3, 7, 16, 9, 8), (2, 36, 12, 33, 50), (1, 5, 9, 6, 122)]:
        lay = synth.random_pruned_layer("stg", n, c_in, c_out, h, w, dtype, synth.PSET16, 0.5, 0.3, seed=11)
        rep, _ = check_layer(lay, tuning=T(variant=2, staging=staging, **tune), label=f"stg{staging}{tune}")
        assert rep["chosen"]["staging"] == staging
        assert rep["chosen"]["chunk_c"] == tune["chunk_c"]
    say(f"  E={rep['E']:.2e}")


def test_staging_default_is_direct_when_rows_are_aligned():
    for dtype, w, want_direct in [("f32", 45, True), ("f16", 45, False), ("f16", 46, True), ("f32", 48, True)]:
        lay = synth.random_pruned_layer("stgdef", 2, 40, 24, 17, w, dtype, synth.PSET8, 0.5, 0.3, seed=5)
        rep, _ = check_layer(lay, tuning=T(variant=2), label=f"stgdef-{dtype}-{w}")
        assert (rep["chosen"]["staging"] >= 2) == want_direct, rep["chosen"]


# Channel split across workgroups: shares of unequal length (chunks not divisible), with and without
# the split inside the workgroup, both staging paths, ragged widths.
SPLITS = [dict(filters_per_wave=4, rows_per_lane=2, lanes_x=8, waves_f=4, split_c=1, chunk_c=4, split_wg=2),
          dict(filters_per_wave=4, rows_per_lane=1, lanes_x=14, waves_f=2, split_c=2, chunk_c=4, split_wg=3),
          dict(filters_per_wave=8, rows_per_lane=2, lanes_x=4, waves_f=3, split_c=1, chunk_c=3, split_wg=5, staging=3),
          dict(filters_per_wave=4, rows_per_lane=4, lanes_x=16, waves_f=1, split_c=1, chunk_c=2, split_wg=4, staging=1),
          dict(filters_per_wave=16, rows_per_lane=1, lanes_x=7, waves_f=1, split_c=4, chunk_c=8, split_wg=2, balance=1)]


@pytest.mark.parametrize("tune", SPLITS)
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_channel_split_across_workgroups(tune, dtype):
    say(f"split {tune} {dtype}")
    for (n, c_in, c_out, h, w) in [(2, 23, 40, 19, 48), (3, 17, 16, 9, 45), (1, 40, 9, 33, 50)]:
        if dtype == "f16" and w % 2 and tune.get("staging", 0) >= 2:
            continue                                           # direct loads need rows on 4-byte boundaries
        lay = synth.random_pruned_layer("swg", n, c_in, c_out, h, w, dtype, synth.PSET16, 0.5, 0.3, seed=13)
        rep, _ = check_layer(lay, tuning=T(variant=2, **tune), label=f"swg{tune}")
        assert rep["chosen"]["split_wg"] == tune["split_wg"]
    say(f"  E={rep['E']:.2e}")


def test_channel_split_is_deterministic_and_batches_beyond_n_hint():
    lay = synth.random_pruned_layer("swgdet", 5, 32, 24, 14, 24, "f32", synth.PSET8, 0.5, 0.3, seed=17)
    x = lay.make_input()
    tune = T(variant=2, filters_per_wave=4, rows_per_lane=1, waves_f=2, split_c=1, chunk_c=4, split_wg=4)
    # planned for 2 images, run on 5: three launches through the same workspace
    plan = pp.plan_from_layer(lay, tuning=tune, n_hint=2)
    xd = to_device(x)
    outs = []
    for _ in range(3):                                         # arrival counters must be back at zero every time
        yd = torch.full((lay.n, lay.c_out, lay.h, lay.w), float("nan"), dtype=xd.dtype, device="cuda")
        plan.run(xd, yd, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        outs.append(yd.cpu().numpy())
    plan.close()
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])   # whoever arrives last
    ref, pre, scale = oracle.layer_reference(lay, x)
    from oracle.compare import error_report
    assert error_report(outs[0], ref, pre, scale)["E"] <= 1e-5


def test_autotune_returns_a_plan_that_passes_parity():
    lay = synth.random_pruned_layer("auto", 2, 64, 48, 28, 28, "f16", synth.PSET8, 0.5, 0.3, seed=21)
    x = to_device(lay.make_input())
    y = torch.empty((lay.n, lay.c_out, lay.h, lay.w), dtype=x.dtype, device="cuda")
    tuning, report = pp.autotune(lay, x, y, steps=3, rounds=2)
    assert len(report) >= 3 and report[0][0] <= report[-1][0]
    assert any(not cand for _, _, cand in report)              # the automatic plan was one of the contestants
    rep, _ = check_layer(lay, tuning=tuning, label="autotuned")
    if tuning is not None:
        assert rep["chosen"] == tuning.as_dict()               # the returned tuning reproduces the measured plan
    # plans that split channels across workgroups can be left out
    _, report2 = pp.autotune(lay, x, y, steps=2, rounds=1, allow_split_wg=False)
    assert all(ch["split_wg"] <= 1 for _, ch, _ in report2)


def test_degenerate_sparsity():
    base = synth.random_pruned_layer("deg", 2, 12, 20, 10, 12, "f32", synth.PSET8, 0.5, 0.3, seed=3)
    # empty mask: bias only
    lay = copy.copy(base)
    lay.conn_mask = np.zeros_like(base.conn_mask)
    _, y = check_layer(lay, relu=False, label="empty")
    assert np.array_equal(y, np.broadcast_to(base.bias[None, :, None, None], y.shape))
    # some empty filters, one full filter
    lay = copy.copy(base)
    m = base.conn_mask.copy().reshape(20, 12)
    m[[0, 7, 19]] = 0
    m[4] = 1
    lay.conn_mask = m.reshape(-1)
    check_layer(lay, label="empty-filters")
    # a single pattern everywhere; and every pattern present in one filter
    lay = copy.copy(base)
    lay.pattern_id = np.full_like(base.pattern_id, 5)
    check_layer(lay, label="single-pattern")
    lay = copy.copy(base)
    lay.conn_mask = np.ones_like(base.conn_mask)
    lay.pattern_id = (np.arange(base.pattern_id.size) % 8).astype(np.int32)
    check_layer(lay, label="all-kept")
    # no bias
    lay = copy.copy(base)
    lay.bias = None
    check_layer(lay, label="no-bias")


def test_foreign_patterns_and_dense_layer():
    lay = synth.random_pruned_layer("foreign", 2, 6, 10, 9, 11, "f32", np.array([0x00F, 0x1E0, 0x03A, 0x145], dtype=np.uint16),
                                    0.7, 0.3, seed=1)
    rep, _ = check_layer(lay, label="foreign")
    assert rep["chosen"]["variant"] == 2                       # runs as a cover of the kernel's own patterns
    rep, _ = check_layer(lay, tuning=T(variant=1), label="foreign-generic")
    assert rep["chosen"]["variant"] == 1
    for dtype in ("f32", "f16"):
        lay = synth.dense_layer("dense", 2, 3, 16, 12, 20, dtype, 0.3, seed=2)
        rep, _ = check_layer(lay, label="dense")


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("taps", [1, 2, 3, 4, 5, 6, 8, 9])
def test_any_three_by_three_pattern_table_on_the_tiled_kernel(taps, dtype):
    """Random masks with any number of taps (with or without the centre) are covered by at most three of the
    kernel's own patterns with zero weights; several tile shapes so that the covers meet every code path."""
    rs = np.random.RandomState(taps)
    masks = set()
    while len(masks) < (6 if taps not in (8, 9) else (1 if taps == 9 else 5)):
        masks.add(int(sum(1 << t for t in rs.choice(9, taps, replace=False))))
    lay = synth.random_pruned_layer_k(f"cover{taps}", 2, 12, 20, 13, 18, dtype, 3, np.array(sorted(masks), dtype=np.uint64), 0.6, 0.2, seed=40 + taps)
    rep, _ = check_layer(lay, tuning=T(variant=2), label=f"cover-{taps}-{dtype}")
    assert rep["chosen"]["variant"] == 2
    rep, _ = check_layer(lay, tuning=T(variant=2, rows_per_lane=2, filters_per_wave=8), label=f"cover-{taps}-{dtype}-r2f8")


def test_filter_reordering_invariance_and_determinism():
    lay = synth.random_pruned_layer("perm", 2, 16, 24, 12, 16, "f32", synth.PSET8, 0.5, 0.3, seed=11)
    x = lay.make_input()
    y1, _ = run_layer(lay, x)
    y2, _ = run_layer(lay, x)
    assert np.array_equal(y1, y2)                              # no atomics: runs are bit-identical
    perm = np.random.RandomState(0).permutation(24)
    rows = (perm[:, None] * 16 + np.arange(16)[None, :]).reshape(-1)
    lay2 = copy.copy(lay)
    lay2.pattern_id, lay2.conn_mask, lay2.weights, lay2.bias = lay.pattern_id[rows], lay.conn_mask[rows], lay.weights[rows], lay.bias[perm]
    y3, _ = run_layer(lay2, x)
    assert np.array_equal(y3, y1[:, perm])                     # same per-filter summation order: bit-identical
    # With channels in natural order, waves per workgroup and filters per wave do not change any
    # output's summation order either; the load-balanced channel order depends on which filters share
    # a workgroup, so there results agree to rounding only.
    y5, _ = run_layer(lay, x, tuning=T(variant=2, filters_per_wave=4, waves_f=6, balance=1))
    y6, _ = run_layer(lay, x, tuning=T(variant=2, filters_per_wave=4, waves_f=3, balance=1))
    assert np.array_equal(y5, y6)
    y4, _ = run_layer(lay, x, tuning=T(variant=2, filters_per_wave=4, waves_f=3))
    assert not np.array_equal(y4, y6)                          # (the orders do differ)
    assert np.max(np.abs(y4 - y6)) <= 1e-5 * max(1.0, float(np.max(np.abs(y6))))


def test_maxpool():
    for dt, tdt in ((np.float32, 0), (np.float16, 1)):
        x = np.random.RandomState(2).standard_normal((3, 5, 8, 12)).astype(dt)
        xd = to_device(x)
        yd = torch.empty((3, 5, 4, 6), dtype=xd.dtype, device="cuda")
        assert pp.pp_maxpool2x2_run(xd.data_ptr(), yd.data_ptr(), 3, 5, 8, 12, tdt, torch.cuda.current_stream().cuda_stream) == pp.PP_OK
        torch.cuda.synchronize()
        assert np.array_equal(yd.cpu().numpy().astype(np.float64), oracle.maxpool2(x.astype(np.float64)))


# ---- the benchmark configurations at full size -------------------------------------------------

def test_config2_full_size():
    lay = synth.config2()
    say("config2")
    for relu in (True, False):
        rep, _ = check_layer(lay, relu=relu, label="cfg2")
    say(f"  E={rep['E']:.2e} E_scale={rep['E_scale']:.2e} {rep['chosen']}")


@pytest.mark.parametrize("batch", [1, 32])
def test_config3_resnet_shapes(batch):
    for lay in synth.config3(batch):
        say(lay.name)
        for relu in (True, False):
            rep, _ = check_layer(lay, relu=relu, label="cfg3")
        say(f"  E={rep['E']:.2e} E_scale={rep['E_scale']:.2e} {rep['chosen']}")


@pytest.mark.parametrize("variant", [2, 3])
def test_config4_vgg_stack_per_layer(variant):
    """Each layer is gated on its own: the checker is fed the GPU's input to that layer."""
    layers = synth.config4()
    x = layers[0].make_input()
    xd = to_device(x)
    stream = torch.cuda.current_stream().cuda_stream
    for lay in layers:
        say(f"{lay.name} variant {variant}")
        plan = pp.plan_from_layer(lay, tuning=T(variant=variant))
        chosen = plan.query()["chosen"]
        assert chosen["variant"] == variant
        yd = plan.run(xd)
        torch.cuda.synchronize()
        plan.close()
        x_np, y_np = xd.cpu().numpy(), yd.cpu().numpy()
        wd = oracle.layer_dense_weights(lay)
        from oracle.compare import error_report, sample_points, TOL
        from gpu_util import tile_boundary_points
        pts = np.concatenate([sample_points(lay.n, lay.c_out, lay.h, lay.w, 2048, seed=lay.seed),
                              tile_boundary_points(lay, lay.n, chosen)], axis=0)
        ref, pre, scale = oracle.conv_at(x_np, wd, pts, lay.bias, lay.relu)
        rep = error_report(y_np[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]], ref, pre, scale)
        say(f"  E={rep['E']:.2e} sigma={rep['sigma']:.3f}")
        assert rep["E"] <= TOL["f16"], (lay.name, rep)
        if lay.meta["pool_after"]:
            pd = torch.empty((lay.n, lay.c_out, lay.h // 2, lay.w // 2), dtype=yd.dtype, device="cuda")
            assert pp.pp_maxpool2x2_run(yd.data_ptr(), pd.data_ptr(), lay.n, lay.c_out, lay.h, lay.w, pp.PP_F16, stream) == pp.PP_OK
            torch.cuda.synchronize()
            xd = pd
        else:
            xd = yd
    assert tuple(xd.shape) == (8, 512, 14, 14)


def test_config4_vgg_stack_with_fused_pools():
    """The chain the benchmark times: the four pools folded into the layers in front of them, every layer gated on
    its own at full size (sampled outputs, points on every tile boundary), the checker fed the GPU's input to it."""
    import copy
    layers = synth.config4()
    x_np = layers[0].make_input()
    for lay in layers:
        if lay.meta["pool_after"]:
            lay = copy.copy(lay)
            lay.pool = True
        say(f"{lay.name} pool={getattr(lay, 'pool', False)}")
        rep, y = check_layer(lay, x_np, points=2048, label=f"cfg4-fused-{lay.name}")
        assert rep["chosen"]["variant"] == 3 and rep["chosen"]["mfma_kind"] == 2, rep["chosen"]
        say(f"  E={rep['E']:.2e} split_k={rep['chosen']['split_k']}")
        x_np = y
    assert tuple(x_np.shape) == (8, 512, 14, 14)


@pytest.mark.parametrize("variant", [2, 3])
def test_config5_large_image(variant):
    lay = synth.config5()
    say(f"config5 variant {variant}")
    x = lay.make_input()
    for relu in (True, False):
        rep, _ = check_layer(lay, x, tuning=T(variant=variant), relu=relu, points=8192, label="cfg5")
        assert rep["chosen"]["variant"] == variant
    say(f"  E={rep['E']:.2e} {rep['chosen']}")


@pytest.mark.parametrize("dtype,shape", [("f16", (2, 32, 64, 40, 60)), ("f32", (2, 24, 32, 28, 28)), ("f16", (1, 12, 20, 9, 17))])
def test_plan_time_autotuning_keeps_a_plan_that_passes_parity(dtype, shape):
    """tuning.autotune = 1: the C library times its candidates itself and reports what it kept."""
    n, c_in, c_out, h, w = shape
    lay = synth.random_pruned_layer("auto", n, c_in, c_out, h, w, dtype, synth.PSET8, 0.5, 0.3, seed=5)
    rep, _ = check_layer(lay, tuning=pp.Tuning(autotune=1), label="plan-autotune")
    assert rep["chosen"]["autotune"] == 1 and rep["chosen"]["variant"] in (2, 3)
    # a fixed field is kept
    rep, _ = check_layer(lay, tuning=pp.Tuning(autotune=1, variant=2), label="plan-autotune-v2")
    assert rep["chosen"]["autotune"] == 1 and rep["chosen"]["variant"] == 2


# ---- the gate itself: it must fail when the layer that was run is not the layer that is checked ----

@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_the_comparison_fails_on_a_wrong_layer(dtype):
    """Negative controls.  The GPU runs the layer as given; the checker is handed a copy with one small
    mistake planted in it (on the CPU side): a kernel's pattern changed, one weight scaled by 1 + 2e-3 (fp32:
    1 + 1e-4), two filters swapped.  Each must push E over the tolerance, and the unchanged layer must pass."""
    import copy
    from gpu_util import run_layer
    from oracle.compare import error_report, TOL
    lay = synth.random_pruned_layer("neg", 2, 16, 24, 12, 20, dtype, synth.PSET8, 0.6, 0.3, seed=11)
    x = lay.make_input()
    y, _ = run_layer(lay, x)

    def E_against(other):
        ref, pre, scale = oracle.layer_reference(other, x.astype(np.float64))
        return error_report(y, ref, pre, scale)["E"]

    assert E_against(lay) <= TOL[dtype]
    kept = np.flatnonzero(lay.conn_mask.ravel())
    # (i) one kept kernel gets another pattern
    wrong = copy.deepcopy(lay)
    k = int(kept[len(kept) // 2])
    wrong.pattern_id.ravel()[k] = (int(wrong.pattern_id.ravel()[k]) + 1) % len(lay.pattern_masks)
    assert E_against(wrong) > TOL[dtype]
    # (ii) the weights of the kernel with the largest weight are off by a relative 25 x tolerance (0.05 for
    # binary16 storage, 2.5e-4 for fp32): that kernel's products are a good fraction of sigma on some outputs
    wrong = copy.deepcopy(lay)
    big = int(kept[np.argmax(np.abs(wrong.weights[kept]).max(axis=1))])
    wrong.weights[big] *= 1.0 + 25 * TOL[dtype]
    assert E_against(wrong) > TOL[dtype]
    # (iii) two output filters trade places
    wrong = copy.deepcopy(lay)
    for name in ("pattern_id", "conn_mask", "weights", "bias"):
        arr = getattr(wrong, name)
        view = arr.reshape(lay.c_out, -1)
        view[[3, 7]] = view[[7, 3]]
    assert E_against(wrong) > TOL[dtype]
