"""Seeded synthetic block-pruned fully-connected layers (paper, section 2.1.2).

A layer is a dense weight matrix W[M][K], a block size (BM, BK), and per block one keep flag per block
row and one per block column.  This module only draws data; it multiplies nothing.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

from . import rng

STREAM_ROWKEEP = 5
STREAM_COLKEEP = 6


@dataclass
class BlockLayer:
    name: str
    m: int
    k: int
    n: int                      # columns of the activation matrix (tokens / pixels)
    bm: int
    bk: int
    dtype: str                  # "f16" (storage; accumulation is fp32) or "f32"
    row_keep: np.ndarray        # uint8 [blocks_m, blocks_k, bm]
    col_keep: np.ndarray        # uint8 [blocks_m, blocks_k, bk]
    weights: np.ndarray         # float32 [m, k] (dense; pruned positions hold values that must never matter)
    bias: Optional[np.ndarray]  # float32 [m] or None
    relu: bool = False
    seed: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def blocks_m(self) -> int:
        return (self.m + self.bm - 1) // self.bm

    @property
    def blocks_k(self) -> int:
        return (self.k + self.bk - 1) // self.bk

    def keep_matrix(self) -> np.ndarray:
        """bool [m, k]: element kept.  Built by broadcasting, not by the loop the checker uses."""
        rk = self.row_keep.astype(bool)[:, :, :, None]          # [bm_blocks, bk_blocks, bm, 1]
        ck = self.col_keep.astype(bool)[:, :, None, :]          # [bm_blocks, bk_blocks, 1, bk]
        full = (rk & ck).transpose(0, 2, 1, 3).reshape(self.blocks_m * self.bm, self.blocks_k * self.bk)
        return full[: self.m, : self.k]

    @property
    def kept_weights(self) -> int:
        return int(np.count_nonzero(self.keep_matrix()))

    @property
    def eff_macs(self) -> int:
        return self.kept_weights * self.n

    @property
    def alg_bytes(self) -> int:
        """Read X once, write Y once, read the kept weights and the bias once."""
        b = 4 if self.dtype == "f32" else 2
        return (self.k + self.m) * self.n * b + self.kept_weights * b + 4 * self.m

    def make_input(self, n: Optional[int] = None) -> np.ndarray:
        """X [k, n] uniform in [-1, 1), in the layer's storage dtype."""
        n = self.n if n is None else n
        np_dt = np.float32 if self.dtype == "f32" else np.float16
        x = rng.chunked(rng.uniform01, self.seed, rng.STREAM_INPUT, self.k * n, np_dt, post=lambda u: 2.0 * u - 1.0)
        return x.reshape(self.k, n)


def random_block_layer(name, m, k, n, bm, bk, dtype, row_keep_frac, col_keep_frac, seed, w_std=None, relu=False,
                       with_bias=True, bias_std=0.01, poison=True) -> BlockLayer:
    """Each block keeps each of its rows with probability row_keep_frac and each of its columns with
    probability col_keep_frac, independently (so some blocks end up empty and some full when the block
    is small).  Weights are N(0, w_std); with `poison`, pruned positions hold large values so that a
    kernel that reads one shows up."""
    blocks_m, blocks_k = (m + bm - 1) // bm, (k + bk - 1) // bk
    nb = blocks_m * blocks_k
    rk = (rng.uniform01(seed, STREAM_ROWKEEP, 0, nb * bm) < row_keep_frac).astype(np.uint8).reshape(blocks_m, blocks_k, bm)
    ck = (rng.uniform01(seed, STREAM_COLKEEP, 0, nb * bk) < col_keep_frac).astype(np.uint8).reshape(blocks_m, blocks_k, bk)
    if w_std is None:
        w_std = 1.0 / np.sqrt(max(1.0, k * row_keep_frac * col_keep_frac))
    w = (rng.chunked(rng.normal01, seed, rng.STREAM_WEIGHT, m * k, np.float64) * w_std).astype(np.float32).reshape(m, k)
    bias = (rng.normal01(seed, rng.STREAM_BIAS, 0, m) * bias_std).astype(np.float32) if with_bias else None
    lay = BlockLayer(name, m, k, n, bm, bk, dtype, rk, ck, w, bias, relu=relu, seed=seed,
                     meta={"row_keep": row_keep_frac, "col_keep": col_keep_frac, "w_std": float(w_std)})
    if poison:
        keep = lay.keep_matrix()
        lay.weights = np.where(keep, lay.weights, np.float32(1000.0)).astype(np.float32)
    return lay


def transformer_block_layer(dtype="f16", seed=2206) -> BlockLayer:
    """A feed-forward projection of transformer size, 4096 x 4096 on 4096 tokens, 64 x 64 blocks, about
    one weight in six kept (the uniform rate of the section's accuracy/latency figure)."""
    return random_block_layer("block_ffn_4096", 4096, 4096, 4096, 64, 64, dtype, 0.41, 0.41, seed, relu=True)
