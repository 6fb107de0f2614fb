"""Host logic of the library, no GPU needed: plan metadata against the checker's reference
ordering (bit-exact), packing round trip, error paths, exported symbols."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import synth
import paper_2206_10620_amd as pp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def check_against_reference(lay, tuning=None):
    plan = pp.plan_from_layer(lay, host_only=True, tuning=tuning)
    info = plan.query()
    p = 1 if lay.dense else len(lay.pattern_masks)
    ref = oracle.plan_ref(lay.c_in, lay.c_out, p, np.zeros_like(lay.pattern_id) if lay.dense else lay.pattern_id,
                          lay.conn_mask)
    assert info["k_kept"] == ref["k_kept"]
    for key in ("perm", "kcount", "pat_off", "kidx", "kpat"):
        assert info[key].dtype == ref[key].dtype and np.array_equal(info[key], ref[key]), key
    assert np.array_equal(info["wpacked"], lay.weights[ref["wsel"]])
    return plan, info


@pytest.mark.parametrize("make", [synth.config1, synth.config2, lambda: synth.config3(1)[2], lambda: synth.config5(h=8, w=8),
                                  lambda: synth.config4(batch=1, hw=16)[0], lambda: synth.config4(batch=1, hw=16)[4]])
def test_plan_metadata_bit_exact(make):
    check_against_reference(make())


def test_plan_metadata_with_empty_and_full_filters_and_seeds():
    for seed in (0, 1, 2):
        lay = synth.random_pruned_layer("p", 1, 37, 29, 9, 9, "f32", synth.PSET16, 0.4, 0.1, seed)
        m = lay.conn_mask.reshape(29, 37)
        m[3] = 0
        m[11] = 1
        _, info = check_against_reference(lay)
        assert info["perm"][0] == 11 and info["perm"][-1] == 3


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("tune", [dict(), dict(filters_per_wave=4, split_c=2, chunk_c=6, waves_f=3),
                                  dict(filters_per_wave=16, rows_per_lane=1, lanes_x=7), dict(split_c=4, chunk_c=8),
                                  dict(split_c=2, chunk_c=4, split_wg=3, waves_f=2), dict(split_c=1, chunk_c=5, split_wg=8, balance=1)])
def test_stream_round_trip(dtype, tune):
    lay = synth.random_pruned_layer("p", 2, 37, 29, 12, 20, dtype, synth.PSET16, 0.4, 0.1, 5)
    t = pp.Tuning(variant=2, **tune)
    plan, info = check_against_reference(lay, t)
    assert info["chosen"]["variant"] == 2
    st, kidx, kpat, w = pp.pp_conv_plan_unpack(plan.handle, info["k_kept"])
    assert st == pp.PP_OK
    assert np.array_equal(kidx, info["kidx"]) and np.array_equal(kpat, info["kpat"])
    want = info["wpacked"] if dtype == "f32" else info["wpacked"].astype(np.float16).astype(np.float32)
    assert np.array_equal(w, want)


def test_foreign_pattern_table_runs_on_the_tiled_kernel_as_a_cover_of_its_own_patterns():
    lay = synth.random_pruned_layer("p", 1, 8, 8, 6, 6, "f32", np.array([0x00F, 0x1E0, 0x03A], dtype=np.uint16), 0.5, 0.1, 0)
    plan, info = check_against_reference(lay)
    assert info["chosen"]["variant"] == 2
    st, *_ = pp.pp_conv_plan_unpack(plan.handle, info["k_kept"])
    assert st == pp.PP_ERR_UNSUPPORTED                     # several stream entries per kernel: no round trip
    pp.plan_from_layer(lay, host_only=True, tuning=pp.Tuning(variant=2)).close()
    gen = pp.plan_from_layer(lay, host_only=True, tuning=pp.Tuning(variant=1))
    assert gen.query()["chosen"]["variant"] == 1           # the generic kernel stays available by name
    gen.close()
    # other kernel sizes and strides still have no tiled form in fp32
    k5 = synth.random_pruned_layer_k("k5", 1, 4, 4, 8, 8, "f32", 5, synth.random_pattern_set(5, 6, 3, 1), 0.5, 0.1, 0)
    p5 = pp.plan_from_layer(k5, host_only=True)
    assert p5.query()["chosen"]["variant"] == 1
    p5.close()


def test_error_paths():
    lay = synth.config1()
    H = pp.PP_FLAG_HOST_ONLY
    args = dict(c_in=lay.c_in, c_out=lay.c_out, h=lay.h, w=lay.w, pattern_masks=lay.pattern_masks,
                pattern_id=lay.pattern_id, conn_mask=lay.conn_mask, weights=lay.weights, bias=lay.bias, flags=H)

    def status(**over):
        a = dict(args)
        a.update(over)
        st, h = pp.pp_conv_plan(**a)
        assert (h is None) == (st != pp.PP_OK)
        if h is not None:
            pp.pp_conv_destroy(h)
        return st

    assert status() == pp.PP_OK
    assert status(bias=None) == pp.PP_OK
    assert status(conn_mask=None) == pp.PP_OK
    assert status(weights=None) == pp.PP_ERR_NULL
    assert status(pattern_id=None) == pp.PP_ERR_NULL
    assert status(pattern_masks=None) == pp.PP_ERR_NULL
    assert status(h=0) == pp.PP_ERR_SHAPE
    assert status(c_in=-1) == pp.PP_ERR_SHAPE
    assert status(pattern_masks=np.array([0x03A, 0x1FF], dtype=np.uint16)) == pp.PP_ERR_PATTERN      # nine taps
    assert status(pattern_masks=np.array([0x03A, 0x007], dtype=np.uint16)) == pp.PP_ERR_PATTERN      # three taps
    assert status(pattern_masks=np.array([0x23A] * 8, dtype=np.uint16)) == pp.PP_ERR_PATTERN         # bit 9 set
    bad = lay.pattern_id.copy()
    bad[np.flatnonzero(lay.conn_mask)[0]] = 8
    assert status(pattern_id=bad) == pp.PP_ERR_PATTERN
    bad = lay.pattern_id.copy()
    bad[np.flatnonzero(lay.conn_mask == 0)[0]] = 99          # ids of removed kernels are never read
    assert status(pattern_id=bad) == pp.PP_OK
    assert status(dtype=7) == pp.PP_ERR_UNSUPPORTED
    assert status(flags=H | 64) == pp.PP_ERR_UNSUPPORTED
    assert status(tuning=pp.Tuning(variant=2, filters_per_wave=5)) == pp.PP_ERR_UNSUPPORTED
    assert status(tuning=pp.Tuning(variant=2, split_c=3, chunk_c=8)) == pp.PP_ERR_UNSUPPORTED
    # a host-only plan cannot run; NULL plan / buffers are rejected; destroy(NULL) is a no-op
    st, h = pp.pp_conv_plan(**args)
    xbytes, ybytes = lay.c_in * lay.h * lay.w * 4, lay.c_out * lay.h * lay.w * 4
    assert pp.pp_conv_run(h, 1 << 20, 2 << 20, 1) == pp.PP_ERR_UNSUPPORTED
    # arguments are validated before anything touches a device: misaligned or overlapping buffers
    assert pp.pp_conv_run(h, (1 << 20) + 4, 2 << 20, 1) == pp.PP_ERR_ALIGN
    assert pp.pp_conv_run(h, 1 << 20, (2 << 20) + 8, 1) == pp.PP_ERR_ALIGN
    assert pp.pp_conv_run(h, 1 << 20, (1 << 20) + xbytes - 16, 1) == pp.PP_ERR_ALIGN      # y starts inside x
    assert pp.pp_conv_run(h, (1 << 20) + ybytes - 16, 1 << 20, 1) == pp.PP_ERR_ALIGN      # x starts inside y
    assert pp.pp_conv_run(h, 1 << 20, (1 << 20) + xbytes, 1) == pp.PP_ERR_UNSUPPORTED     # adjacent is fine
    assert pp.pp_conv_run(h, 1 << 20, 2 << 20, 0) == pp.PP_ERR_SHAPE
    assert pp.pp_conv_run(h, 0, 32, 1) == pp.PP_ERR_NULL
    assert pp.pp_conv_run(None, 16, 32, 1) == pp.PP_ERR_NULL
    assert pp.pp_conv_destroy(h) == pp.PP_OK
    assert pp.pp_conv_destroy(None) == pp.PP_OK
    assert pp.pp_maxpool2x2_run(0, 0, 1, 1, 2, 2, 0) == pp.PP_ERR_NULL
    assert pp.pp_maxpool2x2_run(16, 16, 1, 1, 3, 2, 0) == pp.PP_ERR_SHAPE
    assert pp.pp_status_string(pp.PP_ERR_PATTERN) == "bad pattern mask or id"


def test_staging_choice_and_limits():
    """Input staging: direct loads need rows that start on 4-byte boundaries; the ring must fit in LDS."""
    def chosen(lay, **tune):
        plan = pp.plan_from_layer(lay, host_only=True, tuning=pp.Tuning(variant=2, **tune))
        ch = plan.query()["chosen"]
        plan.close()
        return ch

    def lay(dtype, w, c_in=40):
        return synth.random_pruned_layer("stg", 2, c_in, 24, 17, w, dtype, synth.PSET8, 0.5, 0.3, seed=5)

    assert chosen(lay("f32", 45))["staging"] >= 2          # any fp32 width
    assert chosen(lay("f16", 46))["staging"] >= 2          # even fp16 width
    assert chosen(lay("f16", 45))["staging"] == 1          # odd fp16 width: through registers
    assert chosen(lay("f32", 48), staging=1)["staging"] == 1
    ch = chosen(lay("f32", 48), staging=5, chunk_c=4)
    assert ch["staging"] == 5 and ch["chunk_c"] == 4
    # an automatic ring never has more buffers than there are chunks to put in them
    ch = chosen(lay("f32", 48, c_in=6), chunk_c=4)
    assert ch["staging"] == 2
    with pytest.raises(pp.PPError):
        chosen(lay("f16", 45), staging=2)                   # direct loads impossible
    with pytest.raises(pp.PPError):
        chosen(lay("f32", 48), staging=9)
    assert chosen(lay("f32", 48), chunk_c=8, split_c=1, split_wg=5)["split_wg"] == 5      # 40 channels: 5 chunks
    with pytest.raises(pp.PPError):
        chosen(lay("f32", 48), chunk_c=8, split_c=1, split_wg=6)                       # more shares than chunks
    with pytest.raises(pp.PPError):
        chosen(lay("f32", 48), staging=8, chunk_c=32, lanes_x=16, rows_per_lane=4)   # ring larger than LDS


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "pp_conv.h")).read()
    names = set(re.findall(r"\b(pp_[a-z0-9_]+)\s*\(", header))
    assert {"pp_conv_plan", "pp_conv_run", "pp_conv_destroy", "pp_conv_plan_query", "pp_conv_plan_unpack",
            "pp_maxpool2x2_run", "pp_status_string"} <= names
    lib = ctypes.CDLL(pp.library_path())
    for name in names:
        assert hasattr(lib, name), name


def test_binary16_weight_rounding_matches_checker():
    """The library's own binary16 rounding (host packing) agrees with the checker's on awkward values."""
    vals = np.array([0.1, -0.3, 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 6e-8, 3e-8, 2.0 ** -25, 6.1e-5, 65504.0, 1e-3,
                     -2.0 ** -14, 2.0 ** -14 * (1 - 2.0 ** -12)], dtype=np.float32)
    k = len(vals) // 4
    lay = synth.random_pruned_layer("p", 1, k, 1, 4, 4, "f16", synth.PSET8, 1.0, 0.1, 0)
    lay.weights = vals.reshape(k, 4).copy()
    plan = pp.plan_from_layer(lay, host_only=True, tuning=pp.Tuning(variant=2))
    info = plan.query()
    st, kidx, kpat, w = pp.pp_conv_plan_unpack(plan.handle, info["k_kept"])
    assert st == pp.PP_OK
    want = oracle.widen_f16(oracle.round_f16(info["wpacked"].astype(np.float64))).astype(np.float32)
    assert np.array_equal(w, want)


def test_autotune_request_on_a_host_only_plan_falls_back_to_the_rules():
    lay = synth.random_pruned_layer("auto-host", 1, 16, 16, 12, 12, "f16", synth.PSET8, 0.5, 0.3, seed=1)
    plan = pp.plan_from_layer(lay, host_only=True, tuning=pp.Tuning(autotune=1))
    chosen = plan.query()["chosen"]
    plan.close()
    assert chosen["autotune"] == 0 and chosen["variant"] == 3
    with pytest.raises(pp.PPError):
        pp.plan_from_layer(lay, host_only=True, tuning=pp.Tuning(autotune=2))
