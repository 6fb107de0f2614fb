#!/usr/bin/env python3
"""Throughput of the pattern-pruned 3x3 convolution on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--all] [--no-cpu]

A step is one forward pass of the whole hot path (LDS staging, pattern-specialised
multiply-accumulates, fused bias+ReLU epilogue) over one batch of seeded synthetic input that is
already resident in HBM.  The plan (filter kernel reorder + weight packing) is built once, before
the timed region.  Prints ONE JSON line.

metric  : effective GMAC/s = non-zero multiply-accumulates (4 per kept kernel per output pixel) per second
roofline: the dominant (only) kernel against the FP32 vector-ALU peak of the chip
          (256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2 (packed) x 2.4 GHz = 157.3 TFLOP/s; the library is built
          with packed-FP32 formation disabled, so the reachable ceiling is half of that) -- `achieved`
          counts 2 flop per effective MAC, timed with events on the launch stream.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

# HBM-side traffic of one launch (bytes), from rocprofv3 FETCH_SIZE / WRITE_SIZE scaled by a copy
# kernel of known size; see profiles/k1_tiled_<workload>.md.  Valid only for the kernel revision
# it was measured on: reported as null for any other.
MEASURED_TRAFFIC = {
    "cfg2_vgg_mid": ("k1-2026-11-27-m", 20.43e6),
    "cfg5_enhance_1080p": ("k1-2026-11-27-m", 590.66e6),
    "cfg4_vgg_L6": ("k1-2026-11-27-m", 33.08e6),
}


def workloads():
    import synth
    w = {
        "cfg2_vgg_mid": lambda: synth.config2(),
        "cfg5_enhance_1080p": lambda: synth.config5(),
    }
    for i, (c, hw) in enumerate(synth.RESNET_SHAPES):
        w[f"cfg3_resnet_c{c}_n32"] = (lambda i=i: synth.config3(32)[i])
        w[f"cfg3_resnet_c{c}_n1"] = (lambda i=i: synth.config3(1)[i])
    for i in range(13):
        w[f"cfg4_vgg_L{i + 1}"] = (lambda i=i: synth.config4()[i])
    return w


def time_layer(lay, steps, warmup, tuning=None, autotune=False):
    """Returns dict with per-step times of pp_conv_run on the current stream."""
    import torch
    import paper_2206_10620_amd as pp
    x = torch.from_numpy(lay.make_input()).cuda()
    y = torch.empty((lay.n, lay.c_out, lay.h, lay.w), dtype=x.dtype, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    if autotune and tuning is None:
        tuning, _ = pp.autotune(lay, x, y, stream)
    plan = pp.plan_from_layer(lay, tuning=tuning)
    for _ in range(warmup):
        plan.run(x, y, stream)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        plan.run(x, y, stream)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = ev0.elapsed_time(ev1)
    res = dict(wall_ms_per_step=wall * 1e3 / steps, event_ms_per_step=ev_ms / steps, chosen=plan.query()["chosen"],
               x=x, y=y)
    plan.close()
    return res


def summarize(lay, t):
    sec = t["event_ms_per_step"] * 1e-3
    return dict(workload=lay.name, dtype=lay.dtype, n=lay.n, k_kept=lay.k_kept, eff_gmacs=lay.eff_macs / 1e9,
                alg_mb=lay.alg_bytes / 1e6, us_per_step=t["event_ms_per_step"] * 1e3,
                wall_us_per_step=t["wall_ms_per_step"] * 1e3,
                eff_gmac_per_s=lay.eff_macs / sec / 1e9, alg_gb_per_s=lay.alg_bytes / sec / 1e9,
                frac_fp32_valu=2 * lay.eff_macs / sec / 1e12 / PEAK_FP32_TFLOPS,
                frac_hbm=lay.alg_bytes / sec / 1e9 / PEAK_HBM_GBS, params=t["chosen"])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="cfg2_vgg_mid")
    ap.add_argument("--all", action="store_true", help="also time the other benchmark layers (reported under 'others')")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-baseline leg and the parity check")
    ap.add_argument("--copy-ref-mib", type=int, default=0,
                    help="also launch one plain device copy of this many MiB (a reference dispatch for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--tuning", default="", help="f,r,wf,ks,cc overrides for the timed workload (0 = automatic)")
    ap.add_argument("--autotune", action="store_true",
                    help="pick the parameters of every timed workload by measurement (paper_2206_10620_amd.autotune) "
                         "instead of the plan's own rules; reported under config.params and 'tuned'")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on ONE GPU (no collectives, no sharding); run with --gpus 1")

    import torch
    import paper_2206_10620_amd as pp
    pp.lib()                                   # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.copy_ref_mib > 0:
        src = torch.ones(args.copy_ref_mib * (1 << 20) // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                         # one elementwise copy kernel: reads and writes copy_ref_mib MiB
        torch.cuda.synchronize()
        del src, dst

    table = workloads()
    lay = table[args.workload]()
    tuning = None
    if args.tuning:
        f, r, wf, ks, cc = (int(v) for v in args.tuning.split(","))
        tuning = pp.Tuning(variant=2, filters_per_wave=f, rows_per_lane=r, waves_f=wf, split_c=ks, chunk_c=cc)
    t = time_layer(lay, args.steps, args.warmup, tuning, args.autotune)
    s = summarize(lay, t)
    sec_wall = t["wall_ms_per_step"] * 1e-3

    rev, tbytes = MEASURED_TRAFFIC.get(args.workload, (None, None))
    traffic = tbytes if (rev == pp.KERNEL_REVISION and not args.tuning and not args.autotune) else None

    out = {
        "metric": "effective GMAC/s (nonzero MACs), pattern-pruned 3x3 conv",
        "value": lay.eff_macs / sec_wall / 1e9,
        "unit": "GMAC/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t["wall_ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "tuned": bool(args.autotune),
        "dtype": lay.dtype, "data": "synthetic",
        "config": {"workload": lay.name, "n": lay.n, "c_in": lay.c_in, "c_out": lay.c_out, "h": lay.h, "w": lay.w,
                   "patterns": int(len(lay.pattern_masks)), "k_kept": lay.k_kept, "keep": lay.k_kept / (lay.c_in * lay.c_out),
                   "fused": "bias+relu", "params": t["chosen"]},
        "alg_gb_per_s": s["alg_gb_per_s"], "frac_hbm": s["frac_hbm"],
        "roofline": {"bound": "alu", "achieved": 2 * lay.eff_macs / (t["event_ms_per_step"] * 1e-3) / 1e12,
                     "peak": PEAK_FP32_TFLOPS, "unit": "TFLOP/s",
                     "frac": s["frac_fp32_valu"], "traffic": traffic,
                     "kernel": "k1_tiled", "kernel_us": s["us_per_step"]},
    }

    if not args.no_cpu:
        import oracle
        from oracle.compare import error_report
        x_np = t["x"].cpu().numpy()
        y_np = t["y"].cpu().numpy()
        wd = oracle.layer_dense_weights(lay)
        dense_macs = 9.0 * lay.n * lay.h * lay.w * lay.c_in * lay.c_out
        threads = oracle.binding.default_threads()
        if dense_macs <= 4e9:
            x64 = x_np.astype(np.float64)
            passes = 5
            c0 = time.perf_counter()
            for _ in range(passes):
                ref, pre, scale = oracle.conv(x64, wd, lay.bias, lay.relu, want_pre=True, want_scale=True, threads=threads)
            cpu_s = (time.perf_counter() - c0) / passes
            rep = error_report(y_np, ref, pre, scale)
            frac, sample = 1.0, f"the whole layer, mean of {passes} passes"
        else:
            from oracle.compare import sample_points
            npts = int(min(2e9 / (9.0 * lay.c_in), 4e6))
            pts = sample_points(lay.n, lay.c_out, lay.h, lay.w, npts, seed=0)
            c0 = time.perf_counter()
            ref, pre, scale = oracle.conv_at(np.ascontiguousarray(x_np), wd, pts, lay.bias, lay.relu, threads=threads)
            cpu_s = time.perf_counter() - c0
            rep = error_report(y_np[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]], ref, pre, scale)
            frac = len(pts) / (lay.n * lay.c_out * lay.h * lay.w)
            sample = f"{len(pts)} sampled outputs ({frac:.3%} of the layer)"
        out["cpu_baseline"] = {"value": lay.eff_macs * frac / cpu_s / 1e9, "unit": "GMAC/s", "cores": threads,
                               "kind": "oracle", "sample": sample, "seconds": cpu_s}
        out["max_rel_err"] = rep["E"]

    if args.all:
        others = []
        for name, make in table.items():
            if name == args.workload:
                continue
            l2 = make()
            steps = max(20, min(args.steps, int(0.5 / max(l2.eff_macs / 20e12, 1e-5))))
            t2 = time_layer(l2, steps, max(5, args.warmup // 5), None, args.autotune)
            others.append(summarize(l2, t2))
            del t2
            torch.cuda.empty_cache()
        out["others"] = others

    print(json.dumps(out))


if __name__ == "__main__":
    main()
