"""GPU parity of the matrix-core kernel (variant 3: binary16 storage, zero-filled dense weights on the
MFMA units) against the CPU checker: ragged shapes, forced tile geometries, several filter blocks and
channel chunks, other kernel sizes, stride 2, the fused 2x2 max-pool, pattern tables the vector kernel
has no code for.  Tolerance 2e-3 as for every binary16 result."""
import sys

import numpy as np
import pytest

import synth
import paper_2206_10620_amd as pp
from gpu_util import check_layer

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def T(**kw):
    return pp.Tuning(variant=3, **kw)


SHAPES = [(1, 3, 5, 1, 1), (2, 5, 9, 1, 7), (3, 4, 4, 9, 1), (2, 7, 13, 7, 7), (3, 9, 10, 14, 14), (1, 6, 6, 5, 30),
          (2, 10, 17, 11, 33), (1, 19, 8, 28, 28), (5, 8, 24, 3, 56), (1, 12, 8, 20, 130), (2, 33, 40, 6, 64),
          (2, 40, 70, 17, 24), (1, 16, 64, 16, 64), (3, 17, 129, 9, 8), (1, 64, 64, 40, 72)]


@pytest.mark.parametrize("shape", SHAPES)
def test_ragged_shapes(shape):
    n, c_in, c_out, h, w = shape
    say(f"mfma ragged {shape}")
    lay = synth.random_pruned_layer("ragged", n, c_in, c_out, h, w, "f16", synth.PSET16, 0.6, 0.3, seed=n + w)
    for relu in (True, False):
        rep, _ = check_layer(lay, tuning=T(), relu=relu, label=f"mfma-ragged{shape}")
        assert rep["chosen"]["variant"] == 3
    say(f"  E={rep['E']:.2e} {rep['chosen']}")


TILES = [dict(tile_rows=8, tile_cols=64, tiles_per_wave=4), dict(tile_rows=16, tile_cols=32, tiles_per_wave=4),
         dict(tile_rows=4, tile_cols=64, tiles_per_wave=2), dict(tile_rows=9, tile_cols=28, tiles_per_wave=2),
         dict(tile_rows=36, tile_cols=14, tiles_per_wave=4), dict(tile_rows=1, tile_cols=8, tiles_per_wave=2),
         dict(tile_rows=3, tile_cols=5, tiles_per_wave=2), dict(tile_rows=4, tile_cols=128, tiles_per_wave=4, wg_waves=4),
         dict(tile_rows=5, tile_cols=50, tiles_per_wave=2), dict(tile_rows=64, tile_cols=8, tiles_per_wave=4)]


@pytest.mark.parametrize("tile", TILES)
def test_forced_tile_geometries(tile):
    say(f"mfma tile {tile}")
    for (n, c_in, c_out, h, w) in [(2, 21, 37, 19, 45), (3, 16, 16, 8, 8), (2, 9, 72, 11, 48), (1, 35, 20, 5, 300)]:
        lay = synth.random_pruned_layer("tile", n, c_in, c_out, h, w, "f16", synth.PSET16, 0.5, 0.3, seed=7)
        rep, _ = check_layer(lay, tuning=T(**tile), label=f"mfma-tile{tile}")
        for k, v in tile.items():
            assert rep["chosen"][k] == v
    say(f"  E={rep['E']:.2e}")


@pytest.mark.parametrize("ksize,taps", [(1, 1), (3, 4), (3, 2), (5, 4), (5, 9), (7, 6)])
@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("pool", [False, True])
def test_kernel_sizes_strides_and_fused_pool(ksize, taps, stride, pool):
    say(f"mfma k={ksize} taps={taps} stride={stride} pool={pool}")
    pset = synth.random_pattern_set(ksize, taps, 1 if ksize == 1 else 6, seed=ksize + taps)
    for (n, c_in, c_out, h, w) in [(2, 20, 24, 16, 24), (3, 7, 70, 12, 36), (1, 33, 9, 28, 52), (2, 5, 6, 4, 4)]:
        lay = synth.random_pruned_layer_k("gen", n, c_in, c_out, h, w, "f16", ksize, pset, 0.6, 0.3, seed=3, stride=stride,
                                          pool=pool)
        for relu in (True, False):
            rep, y = check_layer(lay, tuning=T(), relu=relu, label=f"mfma-k{ksize}s{stride}p{int(pool)}")
            assert y.shape[2:] == (lay.out_h, lay.out_w)
    say(f"  E={rep['E']:.2e} {rep['chosen']}")


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("ksize,taps,stride,pool", [(1, 1, 1, False), (3, 4, 2, False), (3, 4, 1, True), (5, 6, 2, True), (7, 5, 1, False)])
def test_generic_kernel_takes_every_layer(dtype, ksize, taps, stride, pool):
    pset = synth.random_pattern_set(ksize, taps, 1 if ksize == 1 else 5, seed=1)
    lay = synth.random_pruned_layer_k("gen0", 2, 9, 11, 12, 16, dtype, ksize, pset, 0.6, 0.3, seed=4, stride=stride, pool=pool)
    for relu in (True, False):
        rep, _ = check_layer(lay, tuning=pp.Tuning(variant=1), relu=relu, label="generic-general")
        assert rep["chosen"]["variant"] == 1
    if dtype == "f32":       # without binary16 storage nothing but the generic kernel takes these layers
        rep, _ = check_layer(lay, label="generic-general-auto")
        assert rep["chosen"]["variant"] == (1 if (ksize != 3 or stride != 1 or pool) else rep["chosen"]["variant"])


def test_any_pattern_table_and_dense_and_degenerate_layers():
    foreign = np.array([0x00F, 0x1E0, 0x03A, 0x145], dtype=np.uint16)
    lay = synth.random_pruned_layer("foreign", 2, 24, 40, 19, 33, "f16", foreign, 0.7, 0.3, seed=1)
    rep, _ = check_layer(lay, label="mfma-foreign")
    assert rep["chosen"]["variant"] == 3                      # the default for binary16 storage
    lay = synth.dense_layer("dense", 2, 3, 16, 12, 20, "f16", 0.3, seed=2)
    rep, _ = check_layer(lay, tuning=T(), label="mfma-dense")
    import copy
    base = synth.random_pruned_layer("deg", 2, 12, 20, 10, 12, "f16", synth.PSET8, 0.5, 0.3, seed=3)
    lay = copy.copy(base)
    lay.conn_mask = np.zeros_like(base.conn_mask)
    _, y = check_layer(lay, tuning=T(), relu=False, label="mfma-empty")
    assert np.array_equal(y, np.broadcast_to(base.bias.astype(np.float16)[None, :, None, None], y.shape))
    lay = copy.copy(base)
    lay.bias = None
    check_layer(lay, tuning=T(), label="mfma-no-bias")


def test_runs_are_bit_identical():
    from gpu_util import run_layer
    lay = synth.random_pruned_layer("det", 2, 48, 80, 21, 40, "f16", synth.PSET8, 0.4, 0.3, seed=9)
    x = lay.make_input()
    y1, _ = run_layer(lay, x, tuning=T())
    y2, _ = run_layer(lay, x, tuning=T())
    assert np.array_equal(y1, y2)


# ---- the direct-load matrix-core kernel (mfma_kind = 2): 3x3, stride 1, channels in whole chunks of 16 ----

def TD(**kw):
    return pp.Tuning(variant=3, mfma_kind=2, **kw)


DIRECT_SHAPES = [(2, 3, 64, 20, 24), (1, 12, 8, 9, 9), (3, 19, 33, 7, 15), (2, 40, 70, 17, 24),      # channel counts padded to whole chunks
                 (1, 16, 5, 1, 1), (2, 16, 9, 1, 7), (3, 32, 64, 9, 1), (2, 16, 13, 7, 7), (3, 48, 10, 14, 14), (1, 16, 6, 5, 30),
                 (2, 32, 17, 11, 31), (1, 16, 8, 28, 28), (5, 16, 24, 3, 56), (1, 16, 70, 20, 130), (2, 32, 40, 6, 61),
                 (2, 64, 129, 17, 29), (1, 16, 64, 16, 60), (3, 16, 8, 9, 15), (1, 64, 64, 40, 72), (2, 16, 4, 33, 2)]


@pytest.mark.parametrize("shape", DIRECT_SHAPES)
def test_direct_ragged_shapes(shape):
    n, c_in, c_out, h, w = shape
    say(f"mfma direct ragged {shape}")
    lay = synth.random_pruned_layer("dragged", n, c_in, c_out, h, w, "f16", synth.PSET16, 0.6, 0.3, seed=n + w)
    for relu in (True, False):
        rep, _ = check_layer(lay, tuning=TD(), relu=relu, label=f"mfma-direct{shape}")
        assert rep["chosen"]["variant"] == 3 and rep["chosen"]["mfma_kind"] == 2
    say(f"  E={rep['E']:.2e} {rep['chosen']}")


@pytest.mark.parametrize("waves,tile_cols", [(4, 30), (4, 60), (4, 14), (4, 28), (4, 56), (8, 30), (8, 60), (8, 14), (8, 28), (8, 56)])
def test_direct_forced_tile_geometries(waves, tile_cols):
    say(f"mfma direct waves {waves} tile_cols {tile_cols}")
    for (n, c_in, c_out, h, w) in [(2, 32, 37, 19, 45), (3, 16, 16, 8, 8), (2, 16, 72, 11, 48), (1, 48, 20, 5, 300), (2, 16, 8, 70, 33)]:
        if waves == 8:
            c_in = max(c_in, 32)            # eight wavefronts stage two chunks ahead: the layer needs at least two
        lay = synth.random_pruned_layer("dtile", n, c_in, c_out, h, w, "f16", synth.PSET16, 0.5, 0.3, seed=7)
        rep, _ = check_layer(lay, tuning=TD(tile_cols=tile_cols, wg_waves=waves), label=f"mfma-direct-tile{waves}x{tile_cols}")
        assert rep["chosen"]["tile_cols"] == tile_cols and rep["chosen"]["mfma_kind"] == 2 and rep["chosen"]["wg_waves"] == waves
    say(f"  E={rep['E']:.2e} {rep['chosen']}")


def test_direct_is_the_default_where_it_applies_and_matches_the_general_kernel():
    from gpu_util import run_layer
    foreign = np.array([0x00F, 0x1E0, 0x03A, 0x145], dtype=np.uint16)
    lay = synth.random_pruned_layer("dauto", 2, 32, 40, 19, 33, "f16", foreign, 0.7, 0.3, seed=1)
    rep, y = check_layer(lay, label="mfma-direct-auto")
    assert rep["chosen"]["variant"] == 3 and rep["chosen"]["mfma_kind"] == 2
    y1, chosen1 = run_layer(lay, lay.make_input(), tuning=pp.Tuning(variant=3, mfma_kind=1))
    assert chosen1["mfma_kind"] == 1
    # same products, summed in a different order: equal to within binary16 output rounding
    assert np.max(np.abs(y.astype(np.float32) - y1.astype(np.float32))) <= 2e-3 * max(1.0, float(np.abs(y1).max()))
    # layers it does not take (another kernel size, a stride, a fused pool) fall to the general kernel; asking for it by name is refused
    lay2 = synth.random_pruned_layer_k("dno", 1, 16, 8, 10, 10, "f16", 3, synth.PSET8, 0.5, 0.3, seed=2, stride=2)
    rep2, _ = check_layer(lay2, tuning=pp.Tuning(variant=3), label="mfma-general-auto")
    assert rep2["chosen"]["mfma_kind"] == 1
    with pytest.raises(pp.PPError):
        pp.plan_from_layer(lay2, tuning=TD())
    # empty filters, no bias, identity activation
    import copy
    lay3 = copy.copy(lay)
    lay3.conn_mask = np.zeros_like(lay.conn_mask)
    _, y3 = check_layer(lay3, tuning=TD(), relu=False, label="mfma-direct-empty")
    assert np.array_equal(y3, np.broadcast_to(lay.bias.astype(np.float16)[None, :, None, None], y3.shape))
    lay4 = copy.copy(lay)
    lay4.bias = None
    check_layer(lay4, tuning=TD(), label="mfma-direct-no-bias")


def test_direct_runs_are_bit_identical():
    from gpu_util import run_layer
    lay = synth.random_pruned_layer("ddet", 2, 48, 80, 21, 40, "f16", synth.PSET8, 0.4, 0.3, seed=9)
    x = lay.make_input()
    y1, _ = run_layer(lay, x, tuning=TD())
    y2, _ = run_layer(lay, x, tuning=TD())
    assert np.array_equal(y1, y2)


# ---- reduction split of the direct-load kernel (tuning.split_k): several workgroups share a tile ----

@pytest.mark.parametrize("waves,split", [(4, 2), (4, 4), (4, 8), (8, 2), (8, 4)])
def test_direct_split_reduction(waves, split):
    say(f"mfma direct split_k {split} waves {waves}")
    # c_in gives 16 or 32 chunks; shapes with several tiles, ragged rows and columns, several filter blocks, a ragged last block
    for (n, c_in, c_out, h, w) in [(2, 256, 40, 9, 13), (3, 512, 130, 14, 14), (1, 256, 64, 5, 61), (2, 256, 8, 17, 3)]:
        lay = synth.random_pruned_layer("dsplit", n, c_in, c_out, h, w, "f16", synth.PSET16, 0.3, 0.1, seed=split + waves)
        for relu in (True, False):
            rep, _ = check_layer(lay, tuning=TD(split_k=split, wg_waves=waves), relu=relu, label=f"mfma-direct-split{split}-w{waves}")
            assert rep["chosen"]["split_k"] == split and rep["chosen"]["mfma_kind"] == 2 and rep["chosen"]["wg_waves"] == waves
    say(f"  E={rep['E']:.2e} {rep['chosen']}")


def test_direct_split_rule_refusals_determinism_and_larger_batches():
    from gpu_util import run_layer
    # few tiles, many chunks: the plan splits by itself
    lay = synth.random_pruned_layer("dsauto", 8, 512, 512, 14, 14, "f16", synth.PSET8, 0.28, 0.03, seed=3)
    rep, y = check_layer(lay, label="mfma-direct-split-auto")
    assert rep["chosen"]["mfma_kind"] == 2 and rep["chosen"]["split_k"] >= 2
    # split off by request gives the same result up to the rounding of a different summation order
    y1, c1 = run_layer(lay, lay.make_input(), tuning=TD(split_k=1))
    assert c1["split_k"] == 1
    assert np.max(np.abs(y.astype(np.float32) - y1.astype(np.float32))) <= 2e-3 * max(1.0, float(np.abs(y1).max()))
    # no atomics: two runs agree bit for bit
    y2, _ = run_layer(lay, lay.make_input())
    assert np.array_equal(y, y2)
    # a plan for 2 images given 5: more than its workspace holds, so it runs unsplit; same gate
    small = synth.random_pruned_layer("dsbig", 5, 256, 64, 7, 7, "f16", synth.PSET8, 0.4, 0.05, seed=4)
    rep, _ = check_layer(small, tuning=TD(split_k=4), n_hint=2, label="mfma-direct-split-beyond-hint")
    assert rep["chosen"]["split_k"] == 4
    # refusals: a share must be whole chunks and at least two of them; only the direct-load kernel splits
    with pytest.raises(pp.PPError):
        pp.plan_from_layer(synth.random_pruned_layer("r1", 1, 48, 8, 8, 8, "f16", synth.PSET8, 0.5, 0.1, seed=1), tuning=TD(split_k=2))
    with pytest.raises(pp.PPError):
        pp.plan_from_layer(synth.random_pruned_layer("r2", 1, 64, 8, 8, 8, "f16", synth.PSET8, 0.5, 0.1, seed=1), tuning=TD(split_k=4))
    with pytest.raises(pp.PPError):
        pp.plan_from_layer(synth.random_pruned_layer("r3", 1, 64, 8, 8, 8, "f16", synth.PSET8, 0.5, 0.1, seed=1), tuning=TD(split_k=3))
    with pytest.raises(pp.PPError):
        pp.plan_from_layer(synth.random_pruned_layer("r4", 1, 64, 8, 8, 8, "f16", synth.PSET8, 0.5, 0.1, seed=1), tuning=pp.Tuning(variant=3, mfma_kind=1, split_k=2))
    with pytest.raises(pp.PPError):
        pp.plan_from_layer(synth.random_pruned_layer("r5", 1, 64, 8, 8, 8, "f32", synth.PSET8, 0.5, 0.1, seed=1), tuning=pp.Tuning(variant=2, split_k=2))


def test_direct_padded_channels_beyond_the_batch_hint_and_dense_first_layer():
    # a plan sized for 2 images given 5: the zero-padded copy of x holds 2, so the batch goes through it in groups
    lay = synth.random_pruned_layer("dpad", 5, 3, 20, 11, 16, "f16", synth.PSET8, 1.0, 0.3, seed=6)
    rep, _ = check_layer(lay, tuning=TD(), n_hint=2, label="mfma-direct-pad-groups")
    assert rep["chosen"]["mfma_kind"] == 2
    # an unpruned three-channel first layer (nine taps) takes the same path by default
    dense = synth.dense_layer("dfirst", 2, 3, 64, 24, 40, "f16", 0.3, seed=2)
    rep, _ = check_layer(dense, label="mfma-direct-dense-first")
    assert rep["chosen"]["variant"] == 3 and rep["chosen"]["mfma_kind"] == 2


# ---- fused 2x2 max-pool on the direct-load kernel ----

@pytest.mark.parametrize("waves", [4, 8])
def test_direct_fused_pool(waves):
    say(f"mfma direct fused pool waves {waves}")
    # even sizes; widths that take 14- and 30-column segments, ragged last segments and tiles, several images and filter blocks,
    # padded channel counts, a ragged last filter block
    for (n, c_in, c_out, h, w) in [(2, 32, 40, 8, 28), (3, 64, 130, 14, 14), (1, 48, 64, 6, 60), (2, 32, 8, 18, 4), (5, 3, 64, 12, 36), (2, 64, 64, 30, 90)]:
        if waves == 8:
            c_in = max(c_in, 32)
        lay = synth.random_pruned_layer_k("dpool", n, c_in, c_out, h, w, "f16", 3, synth.PSET16, 0.5, 0.2, seed=waves + w, pool=True)
        for relu in (True, False):
            rep, _ = check_layer(lay, tuning=TD(wg_waves=waves), relu=relu, label=f"mfma-direct-pool-w{waves}")
            assert rep["chosen"]["mfma_kind"] == 2 and rep["chosen"]["wg_waves"] == waves
    say(f"  E={rep['E']:.2e} {rep['chosen']}")


def test_direct_fused_pool_default_and_refusals():
    lay = synth.random_pruned_layer_k("dpool-auto", 8, 64, 64, 56, 56, "f16", 3, synth.PSET8, 0.28, 0.05, seed=2, pool=True)
    rep, _ = check_layer(lay, label="mfma-direct-pool-auto")
    assert rep["chosen"]["variant"] == 3 and rep["chosen"]["mfma_kind"] == 2
    with pytest.raises(pp.PPError):
        pp.plan_from_layer(lay, host_only=True, tuning=TD(split_k=2))          # partial sums cannot be pooled
    odd = synth.random_pruned_layer_k("dpool-odd", 1, 16, 8, 10, 10, "f16", 3, synth.PSET8, 0.5, 0.1, seed=2, stride=2, pool=False)
    with pytest.raises(pp.PPError):
        pp.plan_from_layer(odd, host_only=True, tuning=TD())


# ---- 1x1 layers as a batch of matrix products on the block-product kernel (mfma_kind 3) ----

def test_pointwise_layers_run_on_the_product_kernel():
    from gpu_util import run_layer
    one = np.array([1], dtype=np.uint16)
    for (n, c_in, c_out, h, w, keep) in [(2, 64, 256, 8, 8, 0.5), (3, 40, 70, 4, 6, 0.6), (1, 256, 64, 56, 56, 0.5), (2, 16, 16, 2, 4, 1.0),
                                          (5, 100, 130, 12, 10, 0.3), (2, 32, 64, 16, 40, 0.0)]:
        lay = synth.random_pruned_layer_k("pw", n, c_in, c_out, h, w, "f16", 1, one, keep, 0.2, seed=n + c_in)
        say(f"pointwise {lay.n}x{c_in}->{c_out} {h}x{w} keep {keep}")
        for relu in (True, False):
            rep, y = check_layer(lay, relu=relu, label="pointwise")
            assert rep["chosen"]["variant"] == 3 and rep["chosen"]["mfma_kind"] == 3, rep["chosen"]
        y1, c1 = run_layer(lay, lay.make_input(), tuning=pp.Tuning(variant=3, mfma_kind=1), relu=False)
        assert c1["mfma_kind"] == 1
        assert np.max(np.abs(y.astype(np.float32) - y1.astype(np.float32))) <= 2e-3 * max(1.0, float(np.abs(y1).max()))
    import copy
    nb = copy.copy(lay)
    nb.bias = None
    nb.conn_mask = np.ones_like(lay.conn_mask)
    check_layer(nb, label="pointwise-no-bias")
    # an image plane that is not a multiple of 8 elements goes to the general kernel; asking for the product kernel there is refused
    odd = synth.random_pruned_layer_k("pw-odd", 2, 32, 32, 7, 7, "f16", 1, one, 0.5, 0.2, seed=3)
    rep, _ = check_layer(odd, label="pointwise-odd")
    assert rep["chosen"]["mfma_kind"] == 1
    with pytest.raises(pp.PPError):
        pp.plan_from_layer(odd, host_only=True, tuning=pp.Tuning(variant=3, mfma_kind=3))
    with pytest.raises(pp.PPError):
        pp.plan_from_layer(synth.random_pruned_layer("pw-3x3", 1, 16, 16, 8, 8, "f16", synth.PSET8, 0.5, 0.2, seed=3), host_only=True,
                           tuning=pp.Tuning(variant=3, mfma_kind=3))
