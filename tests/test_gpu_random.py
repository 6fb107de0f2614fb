"""Randomised parity sweep: seeded shapes x execution parameters, every accepted combination checked
element by element against the checker through the C ABI."""
import random

import pytest

import synth
import paper_2206_10620_amd as pp
from gpu_util import check_layer

pytestmark = pytest.mark.gpu


def _cases(seed, want):
    rng = random.Random(seed)
    out = []
    case = 0
    while len(out) < want:
        case += 1
        n = rng.choice([1, 1, 2, 3, 5])
        c_in = rng.choice([1, 2, 3, 5, 8, 16, 17, 31, 40, 64, 70])
        c_out = rng.choice([1, 3, 4, 7, 8, 16, 33, 64, 70])
        h = rng.choice([1, 2, 3, 7, 8, 13, 14, 28, 33])
        w = rng.choice([1, 2, 3, 4, 7, 8, 14, 15, 16, 28, 30, 31, 56, 64, 66])
        dtype = rng.choice(["f32", "f16"])
        pset = rng.choice([synth.PSET8, synth.PSET16])
        keep = rng.choice([0.1, 0.3, 0.5, 1.0])
        f = rng.choice([4, 4, 8, 16])
        r = rng.choice([1, 2, 4]) if f == 4 else (rng.choice([1, 2]) if f == 8 else 1)
        ks = rng.choice([0, 1, 2, 4, 8])
        tune = dict(filters_per_wave=f, rows_per_lane=r, lanes_x=rng.choice([0, 2, 4, 7, 8, 14, 16]),
                    waves_f=rng.choice([0, 1, 2, 3, 4, 8, 16]), split_c=ks,
                    chunk_c=0 if ks == 0 else rng.choice([0, ks, 2 * ks, 3 * ks, 8 * ks]),
                    staging=rng.choice([0, 0, 1, 2, 3, 4]), split_wg=rng.choice([0, 1, 1, 2, 3]),
                    balance=rng.choice([0, 1, 2]))
        lay = synth.random_pruned_layer("rnd", n, c_in, c_out, h, w, dtype, pset, keep, 0.3, seed=seed * 1000 + case)
        try:
            pp.plan_from_layer(lay, host_only=True, tuning=pp.Tuning(variant=2, **tune)).close()
        except pp.PPError:
            continue                                   # a combination the plan refuses (documented limits)
        out.append((lay, tune))
    return out


@pytest.mark.parametrize("seed", [11, 12])
def test_random_shapes_and_parameters(seed):
    worst = {"f32": 0.0, "f16": 0.0}
    for lay, tune in _cases(seed, 40):
        print(f"n={lay.n} c_in={lay.c_in} c_out={lay.c_out} h={lay.h} w={lay.w} {lay.dtype} {tune}", flush=True)
        rep, _ = check_layer(lay, tuning=pp.Tuning(variant=2, **tune), label=f"rnd{tune}")
        worst[lay.dtype] = max(worst[lay.dtype], rep["E"])
    print(f"worst E: {worst}")
