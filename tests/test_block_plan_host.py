"""Host-side tests of the block-pruned matrix product's plan (no GPU): compact lists against the
checker's masked matrix, packing round trip, error paths, exported symbols."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import synth
import paper_2206_10620_amd as pp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def layers():
    return [
        synth.random_block_layer("a", 128, 128, 16, 64, 64, "f16", 0.5, 0.5, 1),
        synth.random_block_layer("small_blocks", 100, 70, 8, 4, 8, "f16", 0.5, 0.4, 2),
        synth.random_block_layer("big_blocks", 200, 96, 8, 128, 96, "f16", 0.6, 0.3, 3),
        synth.random_block_layer("odd", 65, 33, 8, 7, 5, "f32", 0.5, 0.5, 4),
        synth.random_block_layer("empty", 64, 32, 8, 64, 32, "f16", 0.0, 0.5, 5),
        synth.random_block_layer("full", 70, 40, 8, 16, 16, "f32", 1.0, 1.0, 6),
    ]


@pytest.mark.parametrize("lay", layers(), ids=lambda l: l.name)
def test_lists_and_packed_weights_reproduce_the_masked_matrix(lay):
    plan = pp.block_plan_from_layer(lay, host_only=True)
    try:
        q = plan.query()
        w = lay.weights.astype(np.float64)
        if lay.dtype == "f16":
            w = oracle.widen_f16(oracle.round_f16(w))
        wd = oracle.block_expand(lay.m, lay.k, lay.bm, lay.bk, lay.row_keep, lay.col_keep, w)
        assert q["row_tile"] == 64 and q["row_tiles"] == (lay.m + 63) // 64
        assert q["kept_weights"] == lay.kept_weights
        assert q["variant"] == (2 if lay.dtype == "f16" else 1)
        for t in range(q["row_tiles"]):
            rows = slice(t * 64, min(lay.m, t * 64 + 64))
            off, ln = q["tile_off"][t], q["tile_len"][t]
            cols = q["tile_cols"][off:off + ln]
            assert np.all(np.diff(cols) > 0)
            # every column with a structurally kept weight in the tile is listed, and no column is listed without one
            keep = lay.keep_matrix()[rows]
            assert set(cols.tolist()) == set(np.nonzero(keep.any(axis=0))[0].tolist())
            assert (q["tile_off"][t + 1] - off) % 16 == 0 and 0 <= q["tile_off"][t + 1] - off - ln < 16
            st, dense = pp.pp_block_gemm_unpack(plan.handle, t, 64, lay.k)
            assert st == pp.PP_OK
            want = np.zeros((64, lay.k))
            want[: rows.stop - rows.start] = wd[rows]
            assert np.array_equal(dense.astype(np.float64), want)
        assert q["executed_weights"] == 64 * int(q["tile_off"][-1])
    finally:
        plan.close()


def test_error_paths_need_no_device():
    lay = synth.random_block_layer("e", 64, 64, 8, 32, 32, "f16", 0.5, 0.5, 7)
    H = pp.PP_FLAG_HOST_ONLY
    args = lambda **kw: {**dict(m=64, k=64, block_m=32, block_k=32, row_keep=lay.row_keep, col_keep=lay.col_keep,
                                weights=lay.weights, bias=lay.bias, flags=H, dtype=pp.PP_F16, variant=0), **kw}
    assert pp.pp_block_gemm_plan(**args(weights=None))[0] == pp.PP_ERR_NULL
    assert pp.pp_block_gemm_plan(**args(m=0))[0] == pp.PP_ERR_SHAPE
    assert pp.pp_block_gemm_plan(**args(block_k=0))[0] == pp.PP_ERR_SHAPE
    assert pp.pp_block_gemm_plan(**args(dtype=5))[0] == pp.PP_ERR_UNSUPPORTED
    assert pp.pp_block_gemm_plan(**args(flags=H | 64))[0] == pp.PP_ERR_UNSUPPORTED
    assert pp.pp_block_gemm_plan(**args(variant=3))[0] == pp.PP_ERR_UNSUPPORTED
    assert pp.pp_block_gemm_plan(**args(variant=2, dtype=pp.PP_F32))[0] == pp.PP_ERR_UNSUPPORTED
    st, h = pp.pp_block_gemm_plan(**args())
    assert st == pp.PP_OK
    try:
        # a host-only plan cannot run; argument checks come first
        assert pp.pp_block_gemm_run(h, 0, 4096, 8) == pp.PP_ERR_NULL
        assert pp.pp_block_gemm_run(h, 4096, 1 << 20, 0) == pp.PP_ERR_SHAPE
        assert pp.pp_block_gemm_run(h, 4096 + 2, 1 << 20, 8) == pp.PP_ERR_ALIGN
        assert pp.pp_block_gemm_run(h, 4096, 4096 + 512, 8) == pp.PP_ERR_ALIGN          # overlap
        assert pp.pp_block_gemm_run(h, 4096, 1 << 20, 8) == pp.PP_ERR_UNSUPPORTED
        assert pp.pp_block_gemm_unpack(h, 5, 64, 64)[0] == pp.PP_ERR_SHAPE
    finally:
        pp.pp_block_gemm_destroy(h)
    assert pp.pp_block_gemm_destroy(None) == pp.PP_OK
    # NULL keep arrays mean "all kept"
    st, h = pp.pp_block_gemm_plan(**args(row_keep=None, col_keep=None))
    assert st == pp.PP_OK
    try:
        assert pp.pp_block_gemm_query(h)[1]["kept_weights"] == 64 * 64
    finally:
        pp.pp_block_gemm_destroy(h)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "pp_block_gemm.h")).read()
    names = set(re.findall(r"\b(pp_block_gemm_[a-z0-9_]+)\s*\(", header))
    assert {"pp_block_gemm_plan", "pp_block_gemm_run", "pp_block_gemm_destroy", "pp_block_gemm_query", "pp_block_gemm_unpack"} <= names
    lib = ctypes.CDLL(pp.library_path())
    for name in names:
        assert hasattr(lib, name), name
