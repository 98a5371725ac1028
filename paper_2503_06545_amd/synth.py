"""Seeded synthetic inputs shaped like Open-Sora STDiT linear layers.

This module only draws random tensors.  It holds none of the method's arithmetic
(no quantizer, no GEMM, no reduction) and is the one piece of code that both the
GPU tests/benchmark and the CPU oracle's callers use, so both sides see the same
bits.

Every tensor is addressed by (seed, tensor_id) and generated in row blocks of
ROW_BLOCK rows, each block from its own counter-based Philox stream keyed by
(seed, tensor_id, block index).  Any block of rows can therefore be regenerated on
its own, which is what lets the oracle check sampled rows of the large
configurations without materialising the whole tensor twice.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

ROW_BLOCK = 64

# tensor ids (distinct streams under one seed)
TID_X, TID_W, TID_BIAS, TID_OUTLIER, TID_LATENT_PREV, TID_LATENT_NOISE, TID_MASK = range(1, 8)


def _rng(seed: int, tensor_id: int, block: int) -> np.random.Generator:
    key = np.array([(int(seed) << 32) | int(tensor_id), int(block)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def normal_rows(seed: int, tensor_id: int, row0: int, row1: int, K: int) -> np.ndarray:
    """Rows [row0, row1) of a standard-normal float32 matrix with K columns."""
    out = np.empty((row1 - row0, K), np.float32)
    b0, b1 = row0 // ROW_BLOCK, (row1 + ROW_BLOCK - 1) // ROW_BLOCK
    for b in range(b0, b1):
        blk = _rng(seed, tensor_id, b).standard_normal((ROW_BLOCK, K), dtype=np.float32)
        lo, hi = max(row0, b * ROW_BLOCK), min(row1, (b + 1) * ROW_BLOCK)
        out[lo - row0:hi - row0] = blk[lo - b * ROW_BLOCK:hi - b * ROW_BLOCK]
    return out


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even (a storage cast)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    r = u >> np.uint32(16)          # in-place steps: one temporary instead of five
    r &= np.uint32(1)
    r += np.uint32(0x7FFF)
    r += u
    r >>= np.uint32(16)
    return r.astype(np.uint16)


def outlier_columns(seed: int, K: int, count: int) -> np.ndarray:
    """`count` distinct column indices, a seeded choice."""
    return np.sort(_rng(seed, TID_OUTLIER, 0).choice(K, size=count, replace=False))


def _gelu_tanh_f32(v: np.ndarray) -> np.ndarray:
    # Only shapes the *input distribution* of the fc2 layer (post-GELU activations).
    c = np.float32(math.sqrt(2.0 / math.pi))
    t = v * v
    t *= np.float32(0.044715)
    t += np.float32(1.0)
    t *= v
    t *= c
    np.tanh(t, out=t)
    t += np.float32(1.0)
    t *= v
    t *= np.float32(0.5)
    return t


@dataclass(frozen=True)
class LinearCase:
    """One quantized-linear workload."""
    name: str
    M: int
    K: int
    N: int
    x_dtype: str = "bf16"        # "f32" | "bf16"
    out_dtype: str = "bf16"      # "f32" | "bf16"
    bits: int = 8                # weight bit-width
    epi: str = "none"            # "none" | "gelu_tanh" | "gelu_erf"
    outliers: int = 0            # number of activation columns scaled by 20
    post_gelu: bool = False      # activations are GELU(N(0,1)) (fc2 input)
    seed: int = 0

    def x_rows(self, row0: int, row1: int) -> np.ndarray:
        """Rows of X as float32 (x_dtype f32) or bf16 bit patterns uint16 (x_dtype bf16)."""
        x = normal_rows(self.seed, TID_X, row0, row1, self.K)
        if self.post_gelu:
            x = _gelu_tanh_f32(x)
        if self.outliers:
            cols = outlier_columns(self.seed, self.K, self.outliers)
            x[:, cols] *= np.float32(20.0)
        return to_bf16_bits(x) if self.x_dtype == "bf16" else x

    def x(self) -> np.ndarray:
        """All of X, generated in row chunks (bounded temporaries) on a few threads; the
        chunks are whole row blocks, so the bits do not depend on how the work is split."""
        chunk = 32 * ROW_BLOCK
        starts = range(0, self.M, chunk)
        if len(starts) == 1:
            return self.x_rows(0, self.M)
        out = np.empty((self.M, self.K), np.uint16 if self.x_dtype == "bf16" else np.float32)

        def fill(r):
            out[r:min(self.M, r + chunk)] = self.x_rows(r, min(self.M, r + chunk))

        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
            list(pool.map(fill, starts))
        return out

    def weight(self, layer: int = 0) -> np.ndarray:
        """W float32 [N, K] ~ N(0, std 0.02)."""
        w = normal_rows(self.seed + 1000 * layer, TID_W, 0, self.N, self.K)
        return w * np.float32(0.02)

    def bias(self, layer: int = 0) -> np.ndarray:
        b = normal_rows(self.seed + 1000 * layer, TID_BIAS, 0, 1, self.N)[0]
        return b * np.float32(0.01)


HIDDEN, MLP = 1152, 4608

# the tiny and the single-layer benchmark configurations (the 28-block sweep is built by stdit_block_layers)
TINY = LinearCase("tiny_w8a8", M=256, K=HIDDEN, N=HIDDEN, x_dtype="f32", out_dtype="f32",
                  outliers=8)
QKV_256 = LinearCase("stdit_qkv_256", M=16 * 1024, K=HIDDEN, N=3 * HIDDEN,
                     outliers=round(0.01 * HIDDEN))
FC1_512 = LinearCase("stdit_fc1_gelu_512", M=16 * 4096, K=HIDDEN, N=MLP, epi="gelu_tanh",
                     outliers=round(0.01 * HIDDEN))
FC2_512_W8 = LinearCase("stdit_fc2_512_w8", M=16 * 4096, K=MLP, N=HIDDEN, post_gelu=True)
FC2_512_W4 = LinearCase("stdit_fc2_512_w4", M=16 * 4096, K=MLP, N=HIDDEN, bits=4, post_gelu=True)

LATENT_SHAPE = (16, 4, 16, 64, 64)


def latent_pair(seed: int = 0, n: int | None = None, delta: float = 1e-2):
    """(cur, prev) float32: prev ~ N(0,1), cur = prev + delta * N(0,1)."""
    if n is None:
        n = int(np.prod(LATENT_SHAPE))
    cols = 4096
    rows = (n + cols - 1) // cols
    prev = normal_rows(seed, TID_LATENT_PREV, 0, rows, cols).reshape(-1)[:n].copy()
    noise = normal_rows(seed, TID_LATENT_NOISE, 0, rows, cols).reshape(-1)[:n]
    cur = prev + np.float32(delta) * noise
    return cur.astype(np.float32), prev


def stdit_block_layers(M: int = 2 * 16 * 4096, blocks: int = 28, seed: int = 0, w4_fraction=0.30):
    """The four linears of each of `blocks` STDiT blocks with a seeded per-layer bit-width.

    Layer i is W4 when u_i < w4_fraction, u_i uniform from the seeded mask stream.
    """
    u = _rng(seed, TID_MASK, 0).random(4 * blocks)
    shapes = [("qkv", HIDDEN, 3 * HIDDEN, "none", False), ("out", HIDDEN, HIDDEN, "none", False),
              ("fc1", HIDDEN, MLP, "gelu_tanh", False), ("fc2", MLP, HIDDEN, "none", True)]
    layers = []
    for b in range(blocks):
        for j, (nm, K, N, epi, post) in enumerate(shapes):
            i = 4 * b + j
            layers.append(LinearCase(f"block{b}_{nm}", M=M, K=K, N=N, epi=epi,
                                     bits=4 if u[i] < w4_fraction else 8, post_gelu=post,
                                     outliers=0 if post else round(0.01 * K), seed=seed))
    return layers


def sample_rows(M: int, count: int, tile: int = 256, seed: int = 0) -> np.ndarray:
    """Row indices for sampled parity: first/last rows, rows straddling tile edges, rest random."""
    fixed = {0, 1, M - 1, M - 2}
    for t in range(tile, M, max(tile, (M // 8) // tile * tile or tile)):
        fixed.update((t - 1, t))
    fixed = {r for r in fixed if 0 <= r < M}
    rest = max(0, count - len(fixed))
    rnd = _rng(seed, TID_MASK, 1).choice(M, size=min(M, rest), replace=False)
    rows = np.unique(np.concatenate([np.fromiter(fixed, np.int64), rnd.astype(np.int64)]))
    return rows
