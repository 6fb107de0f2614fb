"""Seeded synthetic layers for deep reuse (paper, section 2.3.2): an activation matrix whose rows resemble each
other, a weight matrix, and the random hyperplanes of the hash.  This module only draws data."""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

from . import rng

STREAM_PROTO = 7
STREAM_PICK = 8
STREAM_HYPER = 9


@dataclass
class ReuseLayer:
    name: str
    n: int
    k: int
    m: int
    seg_len: int
    hash_bits: int
    weights: np.ndarray            # float32 [k, m]
    bias: Optional[np.ndarray]     # float32 [m] or None
    hyperplanes: np.ndarray        # float32 [k // seg_len, hash_bits, seg_len]
    relu: bool = True
    seed: int = 0
    prototypes: int = 64
    noise: float = 0.01
    meta: dict = field(default_factory=dict)

    @property
    def segments(self) -> int:
        return self.k // self.seg_len

    @property
    def dense_macs(self) -> int:
        return self.n * self.k * self.m

    @property
    def alg_bytes(self) -> int:
        """Read x once, write y once, read the weights, hyperplanes and bias once."""
        return 4 * (self.n * (self.k + self.m) + self.k * self.m + self.k * self.hash_bits + self.m)

    def make_input(self, n: Optional[int] = None) -> np.ndarray:
        """x [n, k] float32: every neuron vector is one of `prototypes` random vectors of its segment plus
        N(0, noise) -- the redundancy between positions of an activation map that the method exploits."""
        n = self.n if n is None else n
        S, L = self.segments, self.seg_len
        proto = rng.normal01(self.seed, STREAM_PROTO, 0, S * self.prototypes * L).reshape(S, self.prototypes, L)
        pick = (rng.bits64(self.seed, STREAM_PICK, 0, n * S) % np.uint64(self.prototypes)).astype(np.int64).reshape(n, S)
        x = proto[np.arange(S)[None, :], pick]                                   # [n, S, L]
        x = x + self.noise * rng.chunked(rng.normal01, self.seed, rng.STREAM_INPUT, n * S * L, np.float64).reshape(n, S, L)
        return np.ascontiguousarray(x.reshape(n, self.k).astype(np.float32))


def random_reuse_layer(name, n, k, m, seg_len, hash_bits, seed, prototypes=64, noise=0.01, relu=True, with_bias=True) -> ReuseLayer:
    w = (rng.normal01(seed, rng.STREAM_WEIGHT, 0, k * m) / np.sqrt(k)).astype(np.float32).reshape(k, m)
    b = (rng.normal01(seed, rng.STREAM_BIAS, 0, m) * 0.01).astype(np.float32) if with_bias else None
    hp = rng.normal01(seed, STREAM_HYPER, 0, (k // seg_len) * hash_bits * seg_len).astype(np.float32).reshape(k // seg_len, hash_bits, seg_len)
    return ReuseLayer(name, n, k, m, seg_len, hash_bits, w, b, hp, relu=relu, seed=seed, prototypes=prototypes, noise=noise)


def conv_shaped_reuse_layer(seed=2206) -> ReuseLayer:
    """The unfolded input of a 3x3, 64 -> 64 channel layer on 56 x 56 maps, batch 32: 100 352 rows of 576 values,
    neuron vectors of 16, 12 hash bits, 32 prototypes per segment."""
    return random_reuse_layer("reuse_conv_64x64_56x56_n32", 32 * 56 * 56, 576, 64, 16, 12, seed, prototypes=32)
