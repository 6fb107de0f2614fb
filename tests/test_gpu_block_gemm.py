"""GPU parity of the block-pruned matrix product (paper, section 2.1.2) against the CPU checker, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle.compare import TOL, error_report
import paper_2206_10620_amd as pp

pytestmark = pytest.mark.gpu


def run(lay, x_np, variant=0):
    plan = pp.block_plan_from_layer(lay, variant=variant)
    try:
        xd = torch.from_numpy(np.ascontiguousarray(x_np)).cuda()
        yd = torch.full((lay.m, x_np.shape[1]), float("nan"), dtype=xd.dtype, device="cuda")
        plan.run(xd, yd)
        torch.cuda.synchronize()
        return yd.cpu().numpy(), plan.query()
    finally:
        plan.close()


def check(lay, n=None, variant=0):
    x = lay.make_input(n)
    print(f"case {lay.name} m={lay.m} k={lay.k} n={x.shape[1]} block={lay.bm}x{lay.bk} {lay.dtype} variant={variant}", flush=True)
    got, q = run(lay, x, variant)
    assert not np.isnan(got.astype(np.float64)).any(), "unwritten or invalid outputs"
    ref, pre, sc = oracle.block_layer_reference(lay, x.astype(np.float64))
    rep = error_report(got, ref, pre, sc)
    assert rep["E"] <= TOL[lay.dtype], rep
    return q


# m, k, n, bm, bk, row keep, col keep
SHAPES = [
    (64, 64, 8, 64, 64, 0.5, 0.5),          # one tile, one short chunk list
    (64, 16, 512, 64, 16, 1.0, 1.0),        # a single chunk
    (64, 48, 520, 16, 16, 1.0, 1.0),        # three chunks: exactly the prefetch depth; ragged second column tile
    (64, 80, 64, 16, 16, 1.0, 1.0),         # five chunks: the ring wraps
    (130, 200, 1032, 64, 64, 0.5, 0.5),     # three row tiles (last ragged), three column tiles (last ragged)
    (256, 512, 1024, 4, 16, 0.5, 0.4),      # small blocks: a row tile covers 16 block rows
    (256, 384, 512, 128, 128, 0.4, 0.4),    # blocks larger than a row tile
    (192, 300, 264, 50, 70, 0.6, 0.5),      # block sizes that divide nothing
    (128, 256, 256, 64, 64, 0.0, 0.5),      # every row pruned: bias only
    (128, 256, 256, 64, 64, 0.5, 0.0),      # every column pruned: bias only
]


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(str(v) for v in s[:5]))
def test_matrix_core_kernel_small_shapes(shape, relu):
    m, k, n, bm, bk, rkf, ckf = shape
    lay = synth.random_block_layer("mc", m, k, n, bm, bk, "f16", rkf, ckf, seed=m + k + n, relu=relu)
    q = check(lay)
    assert q["variant"] == 2


def test_no_bias_and_poisoned_pruned_weights():
    lay = synth.random_block_layer("nobias", 128, 256, 512, 32, 32, "f16", 0.5, 0.5, 21, with_bias=False, poison=True)
    check(lay)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("n", [1, 13, 100])
def test_generic_kernel_takes_any_width(dtype, n):
    lay = synth.random_block_layer("gen", 130, 96, n, 16, 32, dtype, 0.5, 0.5, 31 + n, relu=True)
    q = check(lay)
    assert q["variant"] == (2 if dtype == "f16" else 1)      # the plan's kernel for widths that are multiples of 8; these run generic
    if dtype == "f16":
        check(lay, variant=1)


def test_forced_matrix_core_kernel_refuses_other_widths():
    lay = synth.random_block_layer("forced", 64, 64, 12, 32, 32, "f16", 0.5, 0.5, 41)
    plan = pp.block_plan_from_layer(lay, variant=2)
    try:
        x = torch.zeros((64, 12), dtype=torch.float16, device="cuda")
        y = torch.zeros((64, 12), dtype=torch.float16, device="cuda")
        assert pp.pp_block_gemm_run(plan.handle, x.data_ptr(), y.data_ptr(), 12) == pp.PP_ERR_UNSUPPORTED
        assert pp.pp_block_gemm_run(plan.handle, x.data_ptr(), x.data_ptr(), 8) == pp.PP_ERR_ALIGN
    finally:
        plan.close()


def test_both_kernels_agree_with_each_other_through_the_checker():
    lay = synth.random_block_layer("both", 192, 256, 264, 64, 32, "f16", 0.5, 0.5, 51, relu=True)
    check(lay, variant=1)
    check(lay, variant=2)


def test_repeated_runs_are_bit_identical():
    lay = synth.random_block_layer("det", 256, 512, 1024, 64, 64, "f16", 0.41, 0.41, 61, relu=True)
    x = lay.make_input()
    a, _ = run(lay, x)
    b, _ = run(lay, x)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


def test_transformer_sized_layer_at_sampled_outputs():
    """The benchmark's layer at full size; the checker evaluates sampled outputs: random ones, both sides of
    every row-tile and column-tile boundary, the first and last rows and columns."""
    lay = synth.transformer_block_layer()
    x = lay.make_input()
    print(f"case {lay.name} full size", flush=True)
    got, q = run(lay, x)
    assert q["variant"] == 2
    assert not np.isnan(got.astype(np.float32)).any()
    rs = np.random.RandomState(0)
    pts = [np.stack([rs.randint(0, lay.m, 3000), rs.randint(0, lay.n, 3000)], axis=1)]
    rows_edge = sorted({r for b in range(64, lay.m, 64) for r in (b - 1, b)} | {0, lay.m - 1})
    cols_edge = sorted({c for b in range(512, lay.n, 512) for c in (b - 1, b)} | {0, lay.n - 1})
    pts.append(np.stack([np.array(rows_edge)[rs.randint(0, len(rows_edge), 1500)], rs.randint(0, lay.n, 1500)], axis=1))
    pts.append(np.stack([rs.randint(0, lay.m, 1500), np.array(cols_edge)[rs.randint(0, len(cols_edge), 1500)]], axis=1))
    pts = np.concatenate(pts).astype(np.int32)
    w = oracle.widen_f16(oracle.round_f16(lay.weights.astype(np.float64)))
    wd = oracle.block_expand(lay.m, lay.k, lay.bm, lay.bk, lay.row_keep, lay.col_keep, w)
    ref, pre, sc = oracle.gemm_at(wd, x.astype(np.float64), pts, lay.bias, lay.relu)
    rep = error_report(got[pts[:, 0], pts[:, 1]], ref, pre, sc)
    assert rep["E"] <= TOL["f16"], rep


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_the_comparison_fails_on_a_wrong_layer(dtype):
    """Negative controls.  The GPU runs the layer as given; the checker is handed a copy with one mistake planted
    in it on the CPU side: a pruned block row kept, a kept block column pruned, one kept weight off by 25 x the
    tolerance, the row and column flags of the blocks read the other way round.  Each must push E over the
    tolerance, and the unchanged layer must pass."""
    import copy
    lay = synth.random_block_layer("neg", 128, 128, 64, 32, 32, dtype, 0.5, 0.5, 71, poison=False)
    x = lay.make_input()
    got, _ = run(lay, x)

    def E_against(other):
        ref, pre, sc = oracle.block_layer_reference(other, x.astype(np.float64))
        return error_report(got, ref, pre, sc)["E"]

    assert E_against(lay) <= TOL[dtype]
    keep = lay.keep_matrix()
    # a block with kept and pruned rows and columns
    bi, bj = next((i, j) for i in range(lay.blocks_m) for j in range(lay.blocks_k)
                  if 0 < lay.row_keep[i, j].sum() < lay.bm and 0 < lay.col_keep[i, j].sum() < lay.bk)
    wrong = copy.deepcopy(lay)
    wrong.row_keep[bi, bj, int(np.flatnonzero(lay.row_keep[bi, bj] == 0)[0])] = 1
    assert E_against(wrong) > TOL[dtype]
    wrong = copy.deepcopy(lay)
    wrong.col_keep[bi, bj, int(np.flatnonzero(lay.col_keep[bi, bj])[0])] = 0
    assert E_against(wrong) > TOL[dtype]
    wrong = copy.deepcopy(lay)
    r, c = np.unravel_index(int(np.argmax(np.where(keep, np.abs(lay.weights), 0.0))), keep.shape)
    wrong.weights[r, c] *= 1.0 + 25 * TOL[dtype]
    assert E_against(wrong) > TOL[dtype]
    wrong = copy.deepcopy(lay)
    wrong.row_keep, wrong.col_keep = lay.col_keep.copy(), lay.row_keep.copy()       # square blocks: same shapes
    assert E_against(wrong) > TOL[dtype]
