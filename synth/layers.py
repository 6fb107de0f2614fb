"""Seeded synthetic pattern-pruned 3x3 layers shaped like CNN workloads.

A layer is described the way the library's boundary takes it: a table of 9-bit
tap masks (bit t = 3*r + c of the 3x3 window, four bits set), one pattern id
and one keep flag per (output filter, input channel) kernel, four weights per
kept kernel in ascending tap order, and a bias.  The paper prints no pattern
set (its figure of the 4-entry patterns is not reproduced in the text), so the
two sets below are this repository's own stand-ins.

Only data is produced here; no convolution arithmetic lives in this module.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import rng

# ids 0-3: the four T shapes; ids 4-7: the four 2x2 blocks holding the centre.
PSET8 = np.array([0x03A, 0x0B2, 0x0B8, 0x09A, 0x01B, 0x036, 0x0D8, 0x1B0], dtype=np.uint16)
# ids 8-15: diagonal / mixed shapes, all holding the centre tap.
PSET16 = np.concatenate([PSET8, np.array([0x055, 0x115, 0x151, 0x154, 0x152, 0x11C, 0x071, 0x095],
                                         dtype=np.uint16)])


def mask_taps(mask: int) -> List[int]:
    return [t for t in range(9) if (int(mask) >> t) & 1]


@dataclass
class Layer:
    name: str
    n: int
    c_in: int
    c_out: int
    h: int
    w: int
    dtype: str                      # "f32" or "f16": storage type of x, y and packed weights
    pattern_masks: np.ndarray       # uint16 [P]
    pattern_id: np.ndarray          # int32 [c_out*c_in]
    conn_mask: np.ndarray           # uint8 [c_out*c_in]
    weights: np.ndarray             # float32 [c_out*c_in, taps]
    bias: Optional[np.ndarray]      # float32 [c_out] or None
    relu: bool = True
    dense: bool = False             # nine taps per kernel, pattern ids unused
    seed: int = 0
    x_dist: str = "u11"             # "u11" U[-1,1], "u01" U[0,1], "relu_n" max(0, N(0,1))
    meta: dict = field(default_factory=dict)
    ksize: int = 3                  # kernel is ksize x ksize (1, 3, 5 or 7), zero padding (ksize-1)/2
    stride: int = 1                 # 1 or 2
    pool: bool = False              # a 2x2 max-pool (stride 2) follows the activation

    @property
    def taps(self) -> int:
        """Weights stored per kept kernel."""
        return int(self.weights.shape[1])

    @property
    def k_kept(self) -> int:
        return int(np.count_nonzero(self.conn_mask))

    @property
    def conv_h(self) -> int:
        return (self.h - 1) // self.stride + 1

    @property
    def conv_w(self) -> int:
        return (self.w - 1) // self.stride + 1

    @property
    def out_h(self) -> int:
        return self.conv_h // 2 if self.pool else self.conv_h

    @property
    def out_w(self) -> int:
        return self.conv_w // 2 if self.pool else self.conv_w

    @property
    def eff_macs(self) -> int:
        """Nonzero multiply-accumulates of one forward pass."""
        return self.n * self.conv_h * self.conv_w * self.k_kept * self.taps

    @property
    def alg_bytes(self) -> int:
        """Read x once, write y once, read the packed weights (+4 index bytes
        per kept kernel) and the bias once."""
        b = 4 if self.dtype == "f32" else 2
        return (self.n * (self.h * self.w * self.c_in + self.out_h * self.out_w * self.c_out) * b
                + self.k_kept * (self.taps * b + 4) + 4 * self.c_out)

    def make_input(self, n: Optional[int] = None) -> np.ndarray:
        """x [n, c_in, h, w] in the layer's storage dtype."""
        n = self.n if n is None else n
        count = n * self.c_in * self.h * self.w
        np_dt = np.float32 if self.dtype == "f32" else np.float16
        if self.x_dist == "u11":
            x = rng.chunked(rng.uniform01, self.seed, rng.STREAM_INPUT, count, np_dt,
                            post=lambda u: 2.0 * u - 1.0)
        elif self.x_dist == "u01":
            x = rng.chunked(rng.uniform01, self.seed, rng.STREAM_INPUT, count, np_dt)
        elif self.x_dist == "relu_n":
            x = rng.chunked(rng.normal01, self.seed, rng.STREAM_INPUT, count, np_dt,
                            post=lambda g: np.maximum(g, 0.0))
        else:
            raise ValueError(self.x_dist)
        return x.reshape(n, self.c_in, self.h, self.w)


def _round_half_even(v: float) -> int:
    return int(np.rint(v))


def random_pruned_layer(name, n, c_in, c_out, h, w, dtype, pset, keep, w_std, seed,
                        x_dist="u11", relu=True, bias_std=0.01, with_bias=True) -> Layer:
    """Uniform-random pattern per kernel; exactly round(keep*K) kernels kept,
    drawn over the whole layer so per-filter counts vary."""
    k_total = c_in * c_out
    p = len(pset)
    pid = (rng.bits64(seed, rng.STREAM_PATTERN, 0, k_total) % np.uint64(p)).astype(np.int32)
    kept = rng.choose_k(seed, rng.STREAM_CONN, k_total, _round_half_even(keep * k_total))
    conn = np.zeros(k_total, dtype=np.uint8)
    conn[kept] = 1
    wts = (rng.normal01(seed, rng.STREAM_WEIGHT, 0, k_total * 4) * w_std).astype(np.float32).reshape(k_total, 4)
    bias = (rng.normal01(seed, rng.STREAM_BIAS, 0, c_out) * bias_std).astype(np.float32) if with_bias else None
    return Layer(name, n, c_in, c_out, h, w, dtype, np.asarray(pset, dtype=np.uint16), pid, conn, wts, bias,
                 relu=relu, seed=seed, x_dist=x_dist, meta={"keep": keep, "w_std": w_std})


def random_pattern_set(ksize: int, taps: int, count: int, seed: int) -> np.ndarray:
    """`count` distinct (ksize*ksize)-bit masks with `taps` bits each, all holding the centre tap;
    uint64, ascending.  (The paper prints no pattern set for any kernel size.)"""
    kk = ksize * ksize
    centre = kk // 2
    others = [t for t in range(kk) if t != centre]
    found, i = set(), 0
    while len(found) < count:
        pick = rng.choose_k(seed + 7919 * i, rng.STREAM_PATTERN, len(others), taps - 1) if taps > 1 else []
        m = 1 << centre
        for j in pick:
            m |= 1 << others[int(j)]
        found.add(m)
        i += 1
        if i > 100000:
            raise ValueError("not that many patterns exist")
    return np.array(sorted(found), dtype=np.uint64)


def random_pruned_layer_k(name, n, c_in, c_out, h, w, dtype, ksize, pset, keep, w_std, seed, stride=1, pool=False,
                          x_dist="u11", relu=True, bias_std=0.01, with_bias=True) -> Layer:
    """As random_pruned_layer for a ksize x ksize kernel, a stride and an optional fused 2x2 max-pool.
    pset: masks of ksize*ksize bits with the same number of bits each (uint64 for ksize > 3)."""
    pset = np.asarray(pset)
    taps = bin(int(pset[0])).count("1")
    k_total = c_in * c_out
    pid = (rng.bits64(seed, rng.STREAM_PATTERN, 0, k_total) % np.uint64(len(pset))).astype(np.int32)
    kept = rng.choose_k(seed, rng.STREAM_CONN, k_total, _round_half_even(keep * k_total))
    conn = np.zeros(k_total, dtype=np.uint8)
    conn[kept] = 1
    wts = (rng.normal01(seed, rng.STREAM_WEIGHT, 0, k_total * taps) * w_std).astype(np.float32).reshape(k_total, taps)
    bias = (rng.normal01(seed, rng.STREAM_BIAS, 0, c_out) * bias_std).astype(np.float32) if with_bias else None
    masks = pset.astype(np.uint16 if ksize <= 3 else np.uint64)
    return Layer(name, n, c_in, c_out, h, w, dtype, masks, pid, conn, wts, bias, relu=relu, seed=seed, x_dist=x_dist,
                 meta={"keep": keep, "w_std": w_std}, ksize=ksize, stride=stride, pool=pool)


def dense_layer(name, n, c_in, c_out, h, w, dtype, w_std, seed, x_dist="u11", relu=True, bias_std=0.01) -> Layer:
    """Unpruned 3x3 layer: nine weights per kernel, every kernel kept."""
    k_total = c_in * c_out
    wts = (rng.normal01(seed, rng.STREAM_WEIGHT, 0, k_total * 9) * w_std).astype(np.float32).reshape(k_total, 9)
    bias = (rng.normal01(seed, rng.STREAM_BIAS, 0, c_out) * bias_std).astype(np.float32)
    return Layer(name, n, c_in, c_out, h, w, dtype, np.array([0x1FF], dtype=np.uint16),
                 np.zeros(k_total, dtype=np.int32), np.ones(k_total, dtype=np.uint8), wts, bias,
                 relu=relu, dense=True, seed=seed, x_dist=x_dist, meta={"keep": 1.0, "w_std": w_std})


def magnitude_pruned_layer(name, n, c_in, c_out, h, w, dtype, pset, keep_per_filter, seed,
                           x_dist="u11", relu=True, bias_std=0.01) -> Layer:
    """Draw dense N(0,1) 3x3 kernels, then per output filter keep the
    keep_per_filter kernels of largest L2 norm (ties to the lower channel) and
    give each kernel the pattern that retains most of its energy (ties to the
    lower id).  A training-free stand-in for a pruned model."""
    k_total = c_in * c_out
    dense = rng.normal01(seed, rng.STREAM_WEIGHT, 0, k_total * 9).astype(np.float32).reshape(c_out, c_in, 9)
    energy = dense.astype(np.float64) ** 2
    norm2 = energy.sum(axis=2)                                    # [c_out, c_in]
    conn = np.zeros((c_out, c_in), dtype=np.uint8)
    order = np.argsort(-norm2, axis=1, kind="stable")[:, :keep_per_filter]
    np.put_along_axis(conn, order, 1, axis=1)
    tap_lists = np.array([mask_taps(m) for m in pset], dtype=np.int64)       # [P, 4]
    retained = energy[:, :, tap_lists].sum(axis=3)                # [c_out, c_in, P]
    pid = np.argmax(retained, axis=2).astype(np.int32)            # first maximum = lower id
    wts = np.take_along_axis(dense, tap_lists[pid], axis=2)       # [c_out, c_in, 4]
    bias = (rng.normal01(seed, rng.STREAM_BIAS, 0, c_out) * bias_std).astype(np.float32)
    return Layer(name, n, c_in, c_out, h, w, dtype, np.asarray(pset, dtype=np.uint16), pid.reshape(-1),
                 conn.reshape(-1), np.ascontiguousarray(wts.reshape(k_total, 4)), bias, relu=relu, seed=seed,
                 x_dist=x_dist, meta={"keep": keep_per_filter / c_in})


# ---------------------------------------------------------------------------
# The five benchmark configurations
# ---------------------------------------------------------------------------

def _he_std(keep: float, c_in: int, taps: int = 4) -> float:
    """Weight scale that keeps activations O(1): sqrt(2 / effective fan-in)."""
    return float(np.sqrt(2.0 / (taps * keep * c_in)))


def config1(seed: int = 0) -> Layer:
    return random_pruned_layer("cfg1_16x32_32x32", 1, 16, 32, 32, 32, "f32", PSET8, 0.5, 0.1, seed)


def config2(seed: int = 0) -> Layer:
    return magnitude_pruned_layer("cfg2_vgg_mid_256_56x56", 1, 256, 256, 56, 56, "f32", PSET8, 77, seed)


RESNET_SHAPES = [(64, 56), (128, 28), (256, 14), (512, 7)]


def config3(batch: int, seed: int = 0) -> List[Layer]:
    out = []
    for i, (c, hw) in enumerate(RESNET_SHAPES):
        out.append(random_pruned_layer(f"cfg3_resnet_c{c}_{hw}x{hw}_n{batch}", batch, c, c, hw, hw, "f32",
                                       PSET8, 0.5, _he_std(0.5, c), seed + 1000 * i, x_dist="relu_n"))
    return out


VGG16_CHANNELS = [(3, 64), (64, 64), (64, 128), (128, 128), (128, 256), (256, 256), (256, 256),
                  (256, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512)]
VGG16_POOL_AFTER = {2, 4, 7, 10}       # 1-based conv index followed by a 2x2 max-pool


def config4(seed: int = 0, batch: int = 8, hw: int = 224) -> List[Layer]:
    """The 13 conv layers of a VGG-16-shaped stack (pools are the caller's)."""
    layers = []
    size = hw
    for i, (ci, co) in enumerate(VGG16_CHANNELS, start=1):
        s = seed + 1000 * i
        if i == 1:
            lay = dense_layer(f"cfg4_L{i}_dense_{ci}_{co}_{size}", batch, ci, co, size, size, "f16",
                              float(np.sqrt(2.0 / (9 * ci))), s)
        else:
            lay = random_pruned_layer(f"cfg4_L{i}_{ci}_{co}_{size}", batch, ci, co, size, size, "f16", PSET8,
                                      0.28, _he_std(0.28, ci), s)
        lay.meta["pool_after"] = i in VGG16_POOL_AFTER
        layers.append(lay)
        if i in VGG16_POOL_AFTER:
            size //= 2
    return layers


def config5(seed: int = 0, h: int = 1080, w: int = 1920) -> Layer:
    return random_pruned_layer(f"cfg5_enhance_64_{h}x{w}", 1, 64, 64, h, w, "f16", PSET16, 0.4,
                               _he_std(0.4, 64), seed, x_dist="u01")
