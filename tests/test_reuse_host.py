"""Host-side tests of the deep-reuse entry points (no GPU): error paths, exported symbols."""
import ctypes
import os
import re

import numpy as np

import synth
import paper_2206_10620_amd as pp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_error_paths_need_no_device():
    lay = synth.random_reuse_layer("e", 64, 32, 8, 8, 4, 1)
    H = pp.PP_FLAG_HOST_ONLY
    args = lambda **kw: {**dict(k=32, m=8, seg_len=8, hash_bits=4, n_max=64, weights=lay.weights, bias=lay.bias,
                                hyperplanes=lay.hyperplanes, flags=H), **kw}
    assert pp.pp_reuse_plan(**args(weights=None))[0] == pp.PP_ERR_NULL
    assert pp.pp_reuse_plan(**args(hyperplanes=None))[0] == pp.PP_ERR_NULL
    assert pp.pp_reuse_plan(**args(k=0))[0] == pp.PP_ERR_SHAPE
    assert pp.pp_reuse_plan(**args(seg_len=5))[0] == pp.PP_ERR_SHAPE          # does not divide k
    assert pp.pp_reuse_plan(**args(seg_len=64, k=64))[0] == pp.PP_ERR_SHAPE    # neuron vector too long
    assert pp.pp_reuse_plan(**args(hash_bits=0))[0] == pp.PP_ERR_SHAPE
    assert pp.pp_reuse_plan(**args(hash_bits=13))[0] == pp.PP_ERR_SHAPE
    assert pp.pp_reuse_plan(**args(n_max=0))[0] == pp.PP_ERR_SHAPE
    assert pp.pp_reuse_plan(**args(flags=H | 2))[0] == pp.PP_ERR_UNSUPPORTED
    big = synth.random_reuse_layer("big", 8, 4096, 2, 2, 12, 3)
    assert pp.pp_reuse_plan(4096, 2, 2, 12, 8, big.weights, None, big.hyperplanes, H)[0] == pp.PP_ERR_UNSUPPORTED   # hyperplanes beyond LDS
    st, h = pp.pp_reuse_plan(**args(bias=None))
    assert st == pp.PP_OK
    try:
        assert pp.pp_reuse_run(h, 0, 4096, 8) == pp.PP_ERR_NULL
        assert pp.pp_reuse_run(h, 4096, 1 << 20, 0) == pp.PP_ERR_SHAPE
        assert pp.pp_reuse_run(h, 4096, 1 << 20, 65) == pp.PP_ERR_SHAPE        # more rows than the plan was sized for
        assert pp.pp_reuse_run(h, 4096 + 4, 1 << 20, 8) == pp.PP_ERR_ALIGN
        assert pp.pp_reuse_run(h, 4096, 4096 + 64, 8) == pp.PP_ERR_ALIGN       # overlap
        assert pp.pp_reuse_run(h, 4096, 1 << 20, 8) == pp.PP_ERR_UNSUPPORTED   # host-only plan
        assert pp.pp_reuse_read_clusters(h, 8, 4, 4)[0] == pp.PP_ERR_UNSUPPORTED
    finally:
        pp.pp_reuse_destroy(h)
    assert pp.pp_reuse_destroy(None) == pp.PP_OK


def test_synthetic_rows_resemble_each_other():
    lay = synth.random_reuse_layer("s", 400, 32, 4, 8, 6, 2, prototypes=5, noise=0.0)
    x = lay.make_input()
    assert x.shape == (400, 32) and x.dtype == np.float32
    for s in range(4):
        assert len(np.unique(x[:, s * 8:(s + 1) * 8], axis=0)) == 5
    assert np.array_equal(x[:100], lay.make_input(100))                        # a prefix of the same draw


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "pp_deep_reuse.h")).read()
    names = set(re.findall(r"\b(pp_reuse_[a-z0-9_]+)\s*\(", header))
    assert {"pp_reuse_plan", "pp_reuse_run", "pp_reuse_read_clusters", "pp_reuse_destroy"} <= names
    lib = ctypes.CDLL(pp.library_path())
    for name in names:
        assert hasattr(lib, name), name
