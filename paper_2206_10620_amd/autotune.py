"""Pick the execution parameters of a layer by measurement.

The layer-wise representation of the paper has a part that is left to tuning (section 2.3.1); the
plan's own rules choose those parameters from the layer's shape alone.  This helper times a small grid of
alternatives on the device -- rows per lane, channel split inside a workgroup, channel split across
workgroups -- and returns the fastest.  It only builds plans and launches them through the same
entry points as everything else; no arithmetic happens here.

    tuning, report = autotune(layer, x_dev, y_dev)
    plan = plan_from_layer(layer, tuning=tuning)
"""
from __future__ import annotations

import itertools
from typing import Iterable, List, Optional, Tuple

from .pp_conv import PPError, Tuning, plan_from_layer


def default_candidates() -> List[dict]:
    """The automatic choice first; then, for the tiled vector kernel, rows per lane x (split inside, split
    across workgroups); then, for the matrix-core kernel (binary16 layers only), both wavefront tile counts."""
    cands: List[dict] = [dict()]
    for r, (ks, sw) in itertools.product((1, 2), ((1, 1), (2, 1), (4, 1), (1, 2), (2, 2))):
        cands.append(dict(variant=2, filters_per_wave=4, rows_per_lane=r, split_c=ks, split_wg=sw))
    cands.append(dict(variant=3, tiles_per_wave=2))
    cands.append(dict(variant=3, tiles_per_wave=4))
    return cands


def autotune(layer, x_dev, y_dev, stream: Optional[int] = None, steps: int = 20, rounds: int = 3,
             candidates: Optional[Iterable[dict]] = None, allow_split_wg: bool = True) -> Tuple[Optional[Tuning], list]:
    """Time each candidate on (x_dev, y_dev) and return (best tuning or None for the automatic one, report).

    x_dev, y_dev: torch CUDA tensors of the layer's shapes and dtype (y_dev is overwritten).
    report: list of (microseconds per launch, chosen parameters, candidate dict), fastest first.
    allow_split_wg=False leaves out plans that split channels across workgroups (their runs must not
    overlap each other, see the header).
    """
    import torch

    cuda_stream = torch.cuda.current_stream().cuda_stream if stream is None else stream
    plans = []
    seen = set()
    for cand in (default_candidates() if candidates is None else candidates):
        if not allow_split_wg and cand.get("split_wg", 1) > 1:
            continue
        try:
            plan = plan_from_layer(layer, tuning=Tuning(**cand) if cand else None, n_hint=int(x_dev.shape[0]))
        except PPError:
            continue                                    # a candidate this layer cannot run with
        chosen = plan.query()["chosen"]
        key = tuple(sorted(chosen.items()))
        if key in seen:                                 # same plan as an earlier candidate
            plan.close()
            continue
        seen.add(key)
        plans.append((cand, chosen, plan))
    if not plans:
        return None, []
    try:
        for _, _, plan in plans:
            plan.run(x_dev, y_dev, cuda_stream)
        torch.cuda.synchronize()
        best = [float("inf")] * len(plans)
        for _ in range(rounds):                      # candidates take turns, so clock drift hits all alike
            for i, (_, _, plan) in enumerate(plans):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(steps):
                    plan.run(x_dev, y_dev, cuda_stream)
                e1.record()
                torch.cuda.synchronize()
                best[i] = min(best[i], e0.elapsed_time(e1) * 1e3 / steps)
    finally:
        for _, _, plan in plans:
            plan.close()
    report = sorted(((best[i], plans[i][1], plans[i][0]) for i in range(len(plans))), key=lambda t: t[0])
    us, chosen, cand = report[0]
    if not cand:
        return None, report
    fields = {k: v for k, v in chosen.items()}
    return Tuning(**fields), report
