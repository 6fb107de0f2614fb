"""pp_conv_run_static, the run entry point that allocates nothing, against pp_conv_run."""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle.compare import TOL, error_report
import paper_2206_10620_amd as pp

pytestmark = pytest.mark.gpu


def _run_pair(plan, lay, n):
    x = torch.from_numpy(lay.make_input(n)).cuda()
    y0 = torch.full((n, lay.c_out, lay.h, lay.w), float("nan"), dtype=x.dtype, device="cuda")
    y1 = torch.full_like(y0, float("nan"))
    plan.run(x, y0)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    plan.run(x, y1, static=True)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return x.cpu().numpy(), y0.cpu().numpy(), y1.cpu().numpy()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_static_scratch_run_matches_the_allocating_run_twice_in_a_row(dtype):
    lay = synth.random_pruned_layer("noalloc", 4, 64, 48, 14, 20, dtype, synth.PSET8, 0.5, 0.1, seed=5)
    plan = pp.plan_from_layer(lay, tuning=pp.Tuning(variant=2, split_wg=2, chunk_c=16), n_hint=4)
    try:
        assert plan.query()["chosen"]["split_wg"] == 2
        for n in (4, 2):                      # the second call is smaller and finds the first one's leftovers
            x, y0, y1 = _run_pair(plan, lay, n)
            assert not np.isnan(y1.astype(np.float32)).any()
            assert np.array_equal(y0, y1)     # same kernels, same summation order
            ref, pre, scale = oracle.layer_reference(lay, x.astype(np.float64))
            rep = error_report(y1, ref, pre, scale)
            assert rep["E"] <= TOL[dtype], rep
    finally:
        plan.close()


def test_static_scratch_run_without_a_split_and_beyond_the_limit():
    lay = synth.random_pruned_layer("noalloc1", 2, 16, 32, 12, 12, "f32", synth.PSET8, 0.5, 0.1, seed=6)
    plan = pp.plan_from_layer(lay)
    try:
        x, y0, y1 = _run_pair(plan, lay, 2)
        assert np.array_equal(y0, y1)
    finally:
        plan.close()
    # 2 shares x 8 images x 512 filters x 56 x 56 x 4 bytes = 103 MB of partial sums: more than the static buffer
    big = synth.random_pruned_layer("noalloc2", 1, 32, 512, 56, 56, "f32", synth.PSET8, 0.1, 0.1, seed=7)
    plan = pp.plan_from_layer(big, tuning=pp.Tuning(variant=2, split_wg=2, chunk_c=8), n_hint=1)
    try:
        x = torch.zeros((8, 32, 56, 56), dtype=torch.float32, device="cuda")
        y = torch.zeros((8, 512, 56, 56), dtype=torch.float32, device="cuda")
        st = pp.pp_conv_run_static(plan.handle, x.data_ptr(), y.data_ptr(), 8, 0)
        assert st == pp.PP_ERR_SCRATCH
        assert "scratch" in pp.pp_status_string(st)
    finally:
        plan.close()


def test_static_run_of_a_plan_that_splits_its_reduction_runs_unsplit():
    """A matrix-core plan with tuning.split_k > 1 keeps its partial sums in a plan-owned workspace; the entry
    point that allocates nothing does not use it (it runs the same kernel without the split), so its result
    agrees with the allocating run to the rounding of a different summation order, and with the checker."""
    lay = synth.random_pruned_layer("noalloc3", 2, 256, 64, 9, 9, "f16", synth.PSET8, 0.4, 0.05, seed=8)
    plan = pp.plan_from_layer(lay, tuning=pp.Tuning(variant=3, mfma_kind=2, split_k=4), n_hint=2)
    try:
        assert plan.query()["chosen"]["split_k"] == 4
        x, y0, y1 = _run_pair(plan, lay, 2)
        ref, pre, scale = oracle.layer_reference(lay, x.astype(np.float64))
        for y in (y0, y1):
            assert error_report(y, ref, pre, scale)["E"] <= TOL["f16"]
    finally:
        plan.close()
