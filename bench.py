#!/usr/bin/env python3
"""Throughput of the pattern-pruned convolution on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-others] [--no-cpu]

A step is one forward pass of the whole hot path (input staging, multiply-accumulates, fused
bias+ReLU epilogue) over one batch of seeded synthetic input that is already resident in HBM.
The plan (filter kernel reorder + weight packing) is built once, before the timed region.
Prints ONE JSON line.

metric   : effective GMAC/s = non-zero multiply-accumulates (4 per kept kernel per output pixel) per second
workload : by default the largest single-GPU configuration, the 1080p image-enhancement layer (its
           tensors exceed the 256 MB last-level cache, so it streams HBM); every other benchmark layer and
           the VGG-shaped stack run as one chain of launches are timed too and reported under `others`.
roofline : the dominant kernel of the timed workload against the roofline that binds it:
           * the tiled pattern-specialised kernel (variant 2) is bound by the FP32 vector ALUs:
             256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2 (packed) x 2.4 GHz = 157.3 TFLOP/s; the library is
             built with packed-FP32 formation disabled, so `peak_unpacked` = 78.6 TFLOP/s is the reachable
             ceiling.  `achieved` counts 2 flop per effective MAC.
           * the matrix-core kernels (variant 3, zero-filled dense weights in binary16) do 9/(4*keep) times
             the multiply-accumulates at matrix-core rate.  By algorithmic counts the 1080p layer then
             needs 66 us of HBM time (531 MB at 8 TB/s) against 61 us of matrix-core time (153 GFLOP at
             2.5 PFLOP/s): HBM is the binding roofline, and `achieved` = algorithmic bytes (x once, y
             once, packed weights once) per second against 8 TB/s.  The matrix-core fraction (dense flop
             against 2.5 PFLOP/s) is given beside it as `frac_mfma`.
           Kernel time comes from events recorded on the launch stream around the timed launches.
timing   : every timed region follows at least 100 ms of untimed launches of the same work (the chip's clock
           settles some tens of milliseconds into a sustained load).
copy_reference : a plain device copy moving the same activation bytes, timed the same way: what the memory
           system of the box gives the simplest kernel; context for `roofline`, whose peak stays 8 TB/s.
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
PEAK_FP32_UNPACKED_TFLOPS = 78.6
PEAK_MFMA_F16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0

# HBM-side traffic of one launch (bytes), from rocprofv3 FETCH_SIZE / WRITE_SIZE scaled by a copy
# kernel of known size; see profiles/.  Valid only for the kernel revision it was measured on:
# reported as null for any other.  Keyed by (workload, variant).
MEASURED_TRAFFIC = {
    ("cfg5_enhance_1080p", 3): ("lib-2026-11-28-i", 606.92e6),
    ("cfg4_vgg_L6", 3): ("lib-2026-11-28-i", 38.16e6),
    ("cfg4_vgg_L9", 3): ("lib-2026-11-28-i", 53.92e6),
    ("cfg2_vgg_mid", 2): ("lib-2026-11-28-i", 20.43e6),
}

DEFAULT_WORKLOAD = "cfg5_enhance_1080p"


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
    # The fp32 configurations again in binary16 storage (the paper fixes no precision): the same layers, so
    # that the matrix-core path has a number on these shapes too.
    w["cfg2_vgg_mid_f16"] = lambda: _as_f16(synth.config2())
    for i, (c, hw) in enumerate(synth.RESNET_SHAPES):
        w[f"cfg3_resnet_c{c}_n32_f16"] = (lambda i=i: _as_f16(synth.config3(32)[i]))
    # A pattern table that is not the library's own (eight random centre-holding four-tap masks) on the shape of
    # the VGG mid layer: fp32 falls back to the generic kernel, binary16 runs on the matrix cores like any table.
    # The other layer kinds of a ResNet-50-shaped bottleneck stage (section 3's mobile-DSP table): connectivity-pruned
    # 1x1 layers and a pattern-pruned 3x3 layer with stride 2, binary16, batch 32 (general matrix-core kernel).
    w["resnet_1x1_256_64_56_n32"] = lambda: _resnet_kind("resnet_1x1_256_64_56x56_n32", 256, 64, 56, 1, 1)
    w["resnet_1x1_64_256_56_n32"] = lambda: _resnet_kind("resnet_1x1_64_256_56x56_n32", 64, 256, 56, 1, 1)
    w["resnet_3x3s2_128_128_56_n32"] = lambda: _resnet_kind("resnet_3x3s2_128_128_56x56_n32", 128, 128, 56, 3, 2)
    w["cfg2_shape_foreign_patterns_f32"] = lambda: _foreign("f32")
    w["cfg2_shape_foreign_patterns_f16"] = lambda: _foreign("f16")
    return w


def _as_f16(lay):
    lay.dtype = "f16"
    lay.name += "_f16"
    return lay


def _resnet_kind(name, c_in, c_out, hw, ksize, stride):
    import synth
    pset = np.array([1], dtype=np.uint16) if ksize == 1 else synth.PSET8
    taps = 1 if ksize == 1 else 4
    return synth.random_pruned_layer_k(name, 32, c_in, c_out, hw, hw, "f16", ksize, pset, 0.5, float(np.sqrt(2.0 / (taps * 0.5 * c_in))), seed=9,
                                       stride=stride, x_dist="relu_n")


def _foreign(dtype):
    import synth
    own = set(int(m) for m in synth.PSET16)
    masks = [m for m in synth.random_pattern_set(3, 4, 40, seed=11) if int(m) not in own][:8]
    return synth.random_pruned_layer_k(f"cfg2_shape_foreign_patterns_{dtype}", 1, 256, 256, 56, 56, dtype, 3, np.array(masks), 0.3,
                                       float(np.sqrt(2.0 / (4 * 0.3 * 256))), seed=5)


WARM_SECONDS = 0.1     # the clock of this chip settles some tens of milliseconds into a sustained load (the first launches
                       # of the 1080p layer take 222 us, the next few dozen up to 290 us, the sustained ones 210 us): every
                       # timed region is preceded by at least this much untimed work, whatever --warmup says


def _warm(step, warmup):
    """At least `warmup` untimed steps and at least WARM_SECONDS of them."""
    import torch
    t0 = time.perf_counter()
    done = 0
    while done < warmup or time.perf_counter() - t0 < WARM_SECONDS:
        for _ in range(16 if done >= warmup else min(16, warmup - done)):
            step()
            done += 1
        torch.cuda.synchronize()
    return done


def _events():
    import torch
    return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)


def time_layer(lay, steps, warmup, tuning=None, autotune=False):
    """Returns dict with per-step times of pp_conv_run on the current stream."""
    import torch
    import paper_2206_10620_amd as pp
    x = torch.from_numpy(lay.make_input()).cuda()
    y = torch.empty((lay.n, lay.c_out, lay.out_h, lay.out_w), dtype=x.dtype, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    if autotune and tuning is None:
        tuning = pp.Tuning(autotune=1)             # the plan times its candidates itself and keeps the fastest
    plan = pp.plan_from_layer(lay, tuning=tuning)
    _warm(lambda: plan.run(x, y, stream), warmup)
    ev0, ev1 = _events()
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


def time_copy_reference(x, y, layer_us):
    """A plain device-to-device copy that reads as many bytes as the layer's input holds and writes as many as its
    output holds (torch's copy kernel, same warm-up and event timing as the layer): what this machine's memory system
    delivers to the simplest kernel moving the same activation bytes.  Context for `roofline`, not a peak."""
    import torch
    nbytes = (x.numel() * x.element_size() + y.numel() * y.element_size()) // 2
    src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    _warm(lambda: dst.copy_(src), 20)
    ev0, ev1 = _events()
    steps = 50
    ev0.record()
    for _ in range(steps):
        dst.copy_(src)
    ev1.record()
    torch.cuda.synchronize()
    us = ev0.elapsed_time(ev1) * 1e3 / steps
    return {"what": "torch device copy reading and writing as many bytes as the layer's input and output hold",
            "bytes_moved": 2 * (nbytes // 4) * 4, "us": us, "gb_per_s": 2 * (nbytes // 4) * 4 / us / 1e3,
            "layer_us_over_copy_us": layer_us / us}


def dense_macs(lay):
    k = getattr(lay, "ksize", 3)
    return float(k * k) * lay.n * lay.conv_h * lay.conv_w * lay.c_in * lay.c_out


def summarize(lay, t):
    sec = t["event_ms_per_step"] * 1e-3
    return dict(workload=lay.name, dtype=lay.dtype, n=lay.n, k_kept=lay.k_kept, eff_gmacs=lay.eff_macs / 1e9,
                alg_mb=lay.alg_bytes / 1e6, us_per_step=t["event_ms_per_step"] * 1e3,
                wall_us_per_step=t["wall_ms_per_step"] * 1e3,
                eff_gmac_per_s=lay.eff_macs / sec / 1e9, alg_gb_per_s=lay.alg_bytes / sec / 1e9,
                frac_fp32_valu=2 * lay.eff_macs / sec / 1e12 / PEAK_FP32_TFLOPS,
                frac_fp32_valu_unpacked=2 * lay.eff_macs / sec / 1e12 / PEAK_FP32_UNPACKED_TFLOPS,
                frac_mfma_dense=2 * dense_macs(lay) / sec / 1e12 / PEAK_MFMA_F16_TFLOPS,
                frac_hbm=lay.alg_bytes / sec / 1e9 / PEAK_HBM_GBS, params=t["chosen"])


BLOCK_WORKLOAD = "block_ffn_4096"
# HBM-side bytes of one launch of the block-pruned product, measured as above (profiles/k4_block_gemm_block_ffn_4096.md)
MEASURED_TRAFFIC_BLOCK = ("k4-2026-11-28-b", 184.45e6)


def time_block_gemm(steps, warmup, check=True, npts=2000):
    """The block-pruned matrix product (section 2.1.2) on a transformer-sized projection: 4096 x 4096 weights in
    64 x 64 blocks, about one weight in six kept, 4096 columns of activations, binary16 storage.  The matrix
    cores multiply every row of a 64-row tile against the tile's kept columns, so `executed` counts more than
    the kept weights; the roofline of this kernel is the matrix-core one."""
    import torch
    import synth
    import paper_2206_10620_amd as pp
    lay = synth.transformer_block_layer()
    x = torch.from_numpy(lay.make_input()).cuda()
    y = torch.empty((lay.m, lay.n), dtype=x.dtype, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    plan = pp.block_plan_from_layer(lay)
    q = plan.query()
    _warm(lambda: plan.run(x, y, stream), warmup)
    ev0, ev1 = _events()
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        plan.run(x, y, stream)
    ev1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    sec = ev0.elapsed_time(ev1) * 1e-3 / steps
    plan.close()
    executed_flop = 2.0 * q["executed_weights"] * lay.n
    res = dict(workload=lay.name, dtype=lay.dtype, m=lay.m, k=lay.k, n=lay.n, block=[lay.bm, lay.bk],
               kept_weights=int(q["kept_weights"]), executed_weights=int(q["executed_weights"]), kernel="k4_block_gemm" if q["variant"] == 2 else "k4_generic",
               eff_gmacs=lay.eff_macs / 1e9, alg_mb=lay.alg_bytes / 1e6, us_per_step=sec * 1e6, wall_us_per_step=wall * 1e6,
               eff_gmac_per_s=lay.eff_macs / sec / 1e9, alg_gb_per_s=lay.alg_bytes / sec / 1e9,
               executed_tflops=executed_flop / sec / 1e12, frac_mfma_executed=executed_flop / sec / 1e12 / PEAK_MFMA_F16_TFLOPS,
               frac_mfma_effective=2.0 * lay.eff_macs / sec / 1e12 / PEAK_MFMA_F16_TFLOPS, frac_hbm=lay.alg_bytes / sec / 1e9 / PEAK_HBM_GBS)
    if check:
        import oracle
        from oracle.compare import error_report
        rs = np.random.RandomState(0)
        pts = np.stack([rs.randint(0, lay.m, npts), rs.randint(0, lay.n, npts)], axis=1).astype(np.int32)
        w = oracle.widen_f16(oracle.round_f16(lay.weights.astype(np.float64)))
        wd = oracle.block_expand(lay.m, lay.k, lay.bm, lay.bk, lay.row_keep, lay.col_keep, w)
        c0 = time.perf_counter()
        ref, pre, scale = oracle.gemm_at(wd, x.cpu().numpy().astype(np.float64), pts, lay.bias, lay.relu)
        res["cpu_seconds"], res["cpu_outputs"] = time.perf_counter() - c0, npts
        res["max_rel_err"] = error_report(y.cpu().numpy()[pts[:, 0], pts[:, 1]], ref, pre, scale)["E"]
    res["_sec"], res["_wall"], res["_lay"] = sec, wall, lay
    return res


REUSE_WORKLOAD = "reuse_conv_64x64_56x56_n32"


def time_deep_reuse(steps, warmup, check=True):
    """Deep reuse (section 2.3.2) on the unfolded input of a 3x3, 64 -> 64 channel layer, 56 x 56 maps, batch 32
    (100 352 rows of 576 values, binary32): hash + elect representatives, products once per cluster, gather-sum.
    The rate is quoted in dense-equivalent GMAC/s (rows x k x m per second: the product it stands in for);
    the pass is memory-bound, so the roofline is HBM on algorithmic bytes (x once, y once)."""
    import torch
    import synth
    import paper_2206_10620_amd as pp
    lay = synth.conv_shaped_reuse_layer()
    x_np = lay.make_input()
    x = torch.from_numpy(x_np).cuda()
    y = torch.empty((lay.n, lay.m), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    plan = pp.reuse_plan_from_layer(lay)
    _warm(lambda: plan.run(x, y, stream), warmup)
    ev0, ev1 = _events()
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        plan.run(x, y, stream)
    ev1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    sec = ev0.elapsed_time(ev1) * 1e-3 / steps
    sig, rep = plan.clusters(lay.n)
    plan.close()
    clusters = int((rep >= 0).sum())
    res = dict(workload=lay.name, dtype="f32", n=lay.n, k=lay.k, m=lay.m, seg_len=lay.seg_len, hash_bits=lay.hash_bits,
               neuron_vectors=lay.n * lay.segments, clusters=clusters, dense_gmacs=lay.dense_macs / 1e9, alg_mb=lay.alg_bytes / 1e6,
               us_per_step=sec * 1e6, wall_us_per_step=wall * 1e6, dense_equiv_gmac_per_s=lay.dense_macs / sec / 1e9,
               alg_gb_per_s=lay.alg_bytes / sec / 1e9, frac_hbm=lay.alg_bytes / sec / 1e9 / PEAK_HBM_GBS)
    if check:
        import oracle
        from oracle.compare import error_report
        c0 = time.perf_counter()
        ref, pre, scale, rsig, rrep = oracle.reuse_layer(x_np, lay.weights, lay.hyperplanes, lay.seg_len, lay.hash_bits, lay.bias, lay.relu)
        res["cpu_seconds"] = time.perf_counter() - c0
        res["max_rel_err"] = error_report(y.cpu().numpy(), ref, pre, scale)["E"]
        res["clusters_match_checker"] = bool(np.array_equal(sig, rsig) and np.array_equal(rep, rrep))
        exact = np.maximum(x_np.astype(np.float64) @ lay.weights.astype(np.float64) + lay.bias.astype(np.float64), 0.0)
        res["approximation_normwise_vs_exact_product"] = float(np.linalg.norm(ref - exact) / np.linalg.norm(exact))
    res["_sec"], res["_wall"], res["_lay"] = sec, wall, lay
    return res


def reuse_main(args):
    """--workload reuse_conv_64x64_56x56_n32: the JSON line for deep reuse alone (used for its profile)."""
    r = time_deep_reuse(args.steps, max(args.warmup, 10), check=not args.no_cpu)
    sec, wall, lay = r.pop("_sec"), r.pop("_wall"), r.pop("_lay")
    out = {"metric": "dense-equivalent GMAC/s, deep reuse", "value": lay.dense_macs / wall / 1e9, "unit": "GMAC/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {k: r[k] for k in ("workload", "n", "k", "m", "seg_len", "hash_bits", "neuron_vectors", "clusters")},
           "roofline": {"bound": "hbm", "achieved": r["alg_gb_per_s"], "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": r["frac_hbm"],
                        "traffic": None, "kernel": "reuse_hash + reuse_products + reuse_gather", "kernel_us": sec * 1e6}}
    if "max_rel_err" in r:
        import oracle
        out["cpu_baseline"] = {"value": lay.dense_macs / r["cpu_seconds"] / 1e9, "unit": "GMAC/s", "cores": 1, "kind": "oracle",
                               "sample": "the whole layer, one pass", "seconds": r["cpu_seconds"]}
        out["max_rel_err"] = r["max_rel_err"]
        out["clusters_match_checker"] = r["clusters_match_checker"]
        out["approximation_normwise_vs_exact_product"] = r["approximation_normwise_vs_exact_product"]
    print(json.dumps(out))


def block_traffic():
    from paper_2206_10620_amd import pp_block_gemm as pb
    rev, nbytes = MEASURED_TRAFFIC_BLOCK
    return nbytes if rev == pb.BLOCK_KERNEL_REVISION else None


def block_main(args):
    """--workload block_ffn_4096: the JSON line for the block-pruned matrix product alone (used for its profiles)."""
    r = time_block_gemm(args.steps, max(args.warmup, 20), check=not args.no_cpu, npts=2000000)
    sec, wall, lay = r.pop("_sec"), r.pop("_wall"), r.pop("_lay")
    out = {"metric": "effective GMAC/s (nonzero MACs), block-pruned matrix product", "value": lay.eff_macs / wall / 1e9, "unit": "GMAC/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
           "config": {"workload": lay.name, "m": lay.m, "k": lay.k, "n": lay.n, "block": [lay.bm, lay.bk],
                      "kept_weights": r["kept_weights"], "executed_weights": r["executed_weights"], "fused": "bias+relu"},
           "roofline": {"bound": "mfma", "achieved": r["executed_tflops"], "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s",
                        "frac": r["frac_mfma_executed"], "traffic": block_traffic(), "kernel": r["kernel"], "kernel_us": sec * 1e6,
                        "frac_effective": r["frac_mfma_effective"], "frac_hbm": r["frac_hbm"]}}
    if "max_rel_err" in r:
        import oracle
        frac = r["cpu_outputs"] / (lay.m * lay.n)
        out["cpu_baseline"] = {"value": lay.eff_macs * frac / r["cpu_seconds"] / 1e9, "unit": "GMAC/s", "cores": oracle.binding.default_threads(),
                               "kind": "oracle", "sample": f"{r['cpu_outputs']} sampled outputs ({frac:.3%} of the layer)", "seconds": r["cpu_seconds"]}
        out["max_rel_err"] = r["max_rel_err"]
    print(json.dumps(out))


def time_vgg_stack(steps, warmup):
    """The 13 layers of the VGG-shaped configuration as ONE chain on one stream: every plan is built up
    front, every activation buffer is allocated up front, and a step enqueues the 13 convolutions back to
    back with no host synchronisation in between; each layer reads what the previous one wrote.  The four
    2x2 max-pools are folded into the layers in front of them (PP_FLAG_POOL2).  The same chain with the pools
    as separate kernels is timed too (`unfused_us_per_step`), and those pool kernels on their own."""
    import copy
    import torch
    import synth
    import paper_2206_10620_amd as pp
    layers = synth.config4()
    stream = torch.cuda.current_stream().cuda_stream
    x0 = torch.from_numpy(layers[0].make_input()).cuda()

    def build(fused):
        plans, bufs, pools, used = [], [], [], []
        for l in layers:
            pooled = l.meta["pool_after"]
            lf = l
            if pooled and fused:
                lf = copy.copy(l)
                lf.pool = True
            plans.append(pp.plan_from_layer(lf))
            used.append(lf)
            oh, ow = (l.h // 2, l.w // 2) if (pooled and fused) else (l.h, l.w)
            bufs.append(torch.empty((l.n, l.c_out, oh, ow), dtype=torch.float16, device="cuda"))
            pools.append(torch.empty((l.n, l.c_out, l.h // 2, l.w // 2), dtype=torch.float16, device="cuda") if (pooled and not fused) else None)
        return plans, bufs, pools, used

    def pool(i, bufs, pools):
        l = layers[i]
        st = pp.pp_maxpool2x2_run(bufs[i].data_ptr(), pools[i].data_ptr(), l.n, l.c_out, l.h, l.w, pp.PP_F16, stream)
        assert st == pp.PP_OK

    def make_step(plans, bufs, pools):
        def step():
            cur = x0
            for i, plan in enumerate(plans):
                plan.run(cur, bufs[i], stream)
                cur = bufs[i]
                if pools[i] is not None:
                    pool(i, bufs, pools)
                    cur = pools[i]
        return step

    def timed(step):
        _warm(step, warmup)
        ev0, ev1 = _events()
        t0 = time.perf_counter()
        ev0.record()
        for _ in range(steps):
            step()
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / steps, (time.perf_counter() - t0) / steps

    plans, bufs, pools, used = build(True)
    chain_ms, wall = timed(make_step(plans, bufs, pools))
    chosen = [p.query()["chosen"] for p in plans]
    variants = [c["variant"] for c in chosen]
    for p in plans:
        p.close()
    del bufs
    plans_u, bufs_u, pools_u, _ = build(False)
    unfused_ms, _ = timed(make_step(plans_u, bufs_u, pools_u))

    def pools_only():
        for i in range(len(layers)):
            if pools_u[i] is not None:
                pool(i, bufs_u, pools_u)
    pools_ms, _ = timed(pools_only)
    for p in plans_u:
        p.close()
    wall = wall * steps
    eff = sum(l.eff_macs for l in layers)
    alg = sum(l.alg_bytes for l in used)          # pooled layers write a quarter of their outputs
    sec = chain_ms * 1e-3
    return dict(workload="cfg4_vgg_stack_chained", dtype="f16", n=layers[0].n, layers=len(layers), pools=4,
                eff_gmacs=eff / 1e9, alg_mb=alg / 1e6, us_per_step=chain_ms * 1e3, wall_us_per_step=wall * 1e6 / steps,
                pools_us_per_step=pools_ms * 1e3, unfused_us_per_step=unfused_ms * 1e3, fused_pools=True, eff_gmac_per_s=eff / sec / 1e9, alg_gb_per_s=alg / sec / 1e9,
                frac_fp32_valu=2 * eff / sec / 1e12 / PEAK_FP32_TFLOPS,
                frac_fp32_valu_unpacked=2 * eff / sec / 1e12 / PEAK_FP32_UNPACKED_TFLOPS,
                frac_hbm=alg / sec / 1e9 / PEAK_HBM_GBS, variants=variants,
                note="13 convolutions + 4 max-pools enqueued back to back on one stream, no host synchronisation; "
                     "pools_us_per_step is the four pools timed alone")


def roofline_of(lay, t, traffic):
    """The roofline that binds the kernel the plan chose."""
    sec = t["event_ms_per_step"] * 1e-3
    variant = t["chosen"]["variant"]
    if variant == 3:
        return {"bound": "hbm", "achieved": lay.alg_bytes / sec / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": lay.alg_bytes / sec / 1e9 / PEAK_HBM_GBS, "traffic": traffic,
                "kernel": {2: "k3_mfma", 3: "k4_block_gemm"}.get(t["chosen"].get("mfma_kind"), "k2_mfma"),
                "kernel_us": t["event_ms_per_step"] * 1e3,
                "frac_mfma": 2 * dense_macs(lay) / sec / 1e12 / PEAK_MFMA_F16_TFLOPS,
                "peak_mfma_tflops": PEAK_MFMA_F16_TFLOPS}
    ach = 2 * lay.eff_macs / sec / 1e12
    return {"bound": "alu", "achieved": ach, "peak": PEAK_FP32_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_FP32_TFLOPS,
            "traffic": traffic, "kernel": "k1_tiled" if variant == 2 else "k0_generic",
            "kernel_us": t["event_ms_per_step"] * 1e3,
            "peak_unpacked": PEAK_FP32_UNPACKED_TFLOPS, "frac_unpacked": ach / PEAK_FP32_UNPACKED_TFLOPS}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--no-others", action="store_true", help="time only the named workload")
    ap.add_argument("--all", action="store_true", help="(default behaviour; kept for old command lines)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-baseline leg and the parity check")
    ap.add_argument("--copy-ref-mib", type=int, default=0,
                    help="also launch one plain device copy of this many MiB (a reference dispatch for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--tuning", default="", help="f,r,wf,ks,cc overrides for the timed workload (0 = automatic)")
    ap.add_argument("--mfma-tile", default="", help="tile_rows,tile_cols,tiles_per_wave,wg_waves for the matrix-core kernel "
                                                     "on the timed workload (0 = automatic)")
    ap.add_argument("--variant", type=int, default=0, help="force a kernel variant for the timed workload (0 = the plan's choice)")
    ap.add_argument("--autotune", action="store_true",
                    help="let every plan pick its kernel and parameters by measurement (tuning.autotune = 1) "
                         "instead of by its rules; reported under config.params and 'tuned'")
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

    if args.workload == BLOCK_WORKLOAD:
        block_main(args)
        return
    if args.workload == REUSE_WORKLOAD:
        reuse_main(args)
        return
    table = workloads()
    lay = table[args.workload]()
    tuning = None
    if args.tuning:
        f, r, wf, ks, cc = (int(v) for v in args.tuning.split(","))
        tuning = pp.Tuning(variant=2, filters_per_wave=f, rows_per_lane=r, waves_f=wf, split_c=ks, chunk_c=cc)
    elif args.mfma_tile:
        tr, tc, ntw, waves = (int(v) for v in args.mfma_tile.split(","))
        tuning = pp.Tuning(variant=3, tile_rows=tr, tile_cols=tc, tiles_per_wave=ntw, wg_waves=waves)
    elif args.variant:
        tuning = pp.Tuning(variant=args.variant)
    t = time_layer(lay, args.steps, max(args.warmup, 20), tuning, args.autotune)
    s = summarize(lay, t)
    sec_wall = t["wall_ms_per_step"] * 1e-3

    rev, tbytes = MEASURED_TRAFFIC.get((args.workload, t["chosen"]["variant"]), (None, None))
    traffic = tbytes if (rev == pp.KERNEL_REVISION and not args.tuning and not args.mfma_tile and not args.autotune) else None

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
        "frac_fp32_valu": s["frac_fp32_valu"], "frac_fp32_valu_unpacked": s["frac_fp32_valu_unpacked"],
        "roofline": roofline_of(lay, t, traffic),
    }

    out["copy_reference"] = time_copy_reference(t["x"], t["y"], t["event_ms_per_step"] * 1e3)

    if not args.no_cpu:
        import oracle
        from oracle.compare import error_report
        x_np = t["x"].cpu().numpy()
        y_np = t["y"].cpu().numpy()
        wd = oracle.layer_dense_weights(lay)
        threads = oracle.binding.default_threads()
        if dense_macs(lay) <= 4e9:
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
    del t
    torch.cuda.empty_cache()

    if not args.no_others:
        others = []
        for name, make in table.items():
            if name == args.workload:
                continue
            l2 = make()
            steps = max(20, min(200, int(0.2 / max(l2.eff_macs / 20e12, 1e-5))))
            t2 = time_layer(l2, steps, 20, None, args.autotune)
            others.append(summarize(l2, t2))
            del t2
            torch.cuda.empty_cache()
        others.append(time_vgg_stack(steps=20, warmup=5))
        blk = time_block_gemm(steps=50, warmup=10, check=not args.no_cpu)
        others.append({k: v for k, v in blk.items() if not k.startswith("_")})
        del blk
        torch.cuda.empty_cache()
        reu = time_deep_reuse(steps=20, warmup=5, check=not args.no_cpu)
        others.append({k: v for k, v in reu.items() if not k.startswith("_")})
        out["others"] = others

    print(json.dumps(out))


if __name__ == "__main__":
    main()
