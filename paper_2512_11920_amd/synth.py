"""Seeded synthetic KV caches and decode-step access patterns.

This module holds no codec arithmetic: it only draws random FP16 tensors and index arrays with the
shapes and value distribution of the workloads (LLaMA-2-shaped K/V caches, Section 4.1 of the
paper), standing in for caches the paper's models would produce.  Both the CPU-side checker's tests and
the GPU path's tests/benchmark take their inputs from here.

Distribution: for every (layer, K|V, head, channel) a scale c ~ LogNormal(0, 0.5), constant over
tokens and sequences; for K only, each channel is an outlier with probability 0.02 and gets
c * 10; element = N(0,1) * c, rounded to FP16.

Layout of a cache tensor: [layer][K|V][block][head][N][d] ("kv-major", configs 1-4), or
[layer][block][K|V][head][N][d] ("block-major", the decode-gather config, where one logical block
carries the K and V pages of all heads).  block = 16 consecutive tokens of one sequence.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

TAG_SCALE, TAG_OUTLIER, TAG_ELEM, TAG_LEN, TAG_PERM, TAG_PRED = 1, 2, 3, 4, 5, 6


@dataclass(frozen=True)
class KVShape:
    name: str
    n_layers: int
    n_kv_heads: int
    head_dim: int
    seq_len: int
    batch: int
    tokens_per_block: int = 16
    seed: int = 0

    @property
    def blocks_per_layer(self) -> int:  # per K or V
        return self.batch * (self.seq_len // self.tokens_per_block)

    @property
    def page_elems(self) -> int:
        return self.tokens_per_block * self.head_dim

    @property
    def pages_per_layer(self) -> int:  # K and V
        return 2 * self.blocks_per_layer * self.n_kv_heads

    @property
    def n_pages(self) -> int:
        return self.n_layers * self.pages_per_layer

    @property
    def nbytes(self) -> int:
        return self.n_pages * self.page_elems * 2


CONFIGS = {
    "tiny": KVShape("tiny", 1, 4, 64, 256, 1),
    "7b_layer": KVShape("7b_layer", 1, 32, 128, 2048, 8),
    "7b_full": KVShape("7b_full", 32, 32, 128, 2048, 32),
    "70b_gqa": KVShape("70b_gqa", 80, 8, 128, 4096, 16),
}


def _rng(seed: int, tag: int, *idx: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, tag, *idx]))


def channel_scales(shape: KVShape, layer: int) -> np.ndarray:
    """float32 [2 (K,V)][head][d] per-channel multipliers of one layer."""
    c = np.exp(0.5 * _rng(shape.seed, TAG_SCALE, layer).standard_normal((2, shape.n_kv_heads, shape.head_dim)))
    outlier = _rng(shape.seed, TAG_OUTLIER, layer).random((shape.n_kv_heads, shape.head_dim)) < 0.02
    c[0][outlier] *= 10.0
    return c.astype(np.float32)


def layer_numpy(shape: KVShape, layer: int) -> np.ndarray:
    """One layer on the host: float16 [2][blocks][head][N][d] (kv-major)."""
    c = channel_scales(shape, layer)
    g = _rng(shape.seed, TAG_ELEM, layer)
    z = g.standard_normal((2, shape.blocks_per_layer, shape.n_kv_heads, shape.tokens_per_block, shape.head_dim),
                          dtype=np.float32)
    return (z * c[:, None, :, None, :]).astype(np.float16)


def cache_numpy(shape: KVShape) -> np.ndarray:
    """Whole cache on the host: float16 [layer][2][blocks][head][N][d]."""
    return np.stack([layer_numpy(shape, l) for l in range(shape.n_layers)])


def layer_torch(shape: KVShape, layer: int, device, block_major: bool = False, n_blocks: int | None = None):
    """One layer drawn on ``device`` with torch's generator (a different stream from
    layer_numpy, same distribution).  float16 [2][blocks][head][N][d], or
    [blocks][2][head][N][d] when block_major."""
    import torch

    nb = shape.blocks_per_layer if n_blocks is None else n_blocks
    c = torch.from_numpy(channel_scales(shape, layer)).to(device)
    gen = torch.Generator(device=device)
    gen.manual_seed((shape.seed * 1000003 + layer) * 7 + TAG_ELEM)
    H, N, d = shape.n_kv_heads, shape.tokens_per_block, shape.head_dim
    if block_major:
        z = torch.randn((nb, 2, H, N, d), generator=gen, device=device, dtype=torch.float32)
        z.mul_(c[None, :, :, None, :])
    else:
        z = torch.randn((2, nb, H, N, d), generator=gen, device=device, dtype=torch.float32)
        z.mul_(c[:, None, :, None, :])
    return z.to(torch.float16)


def cache_torch(shape: KVShape, device):
    """Whole cache on ``device``, drawn one layer at a time: float16 [layer][2][blocks][head][N][d]."""
    import torch

    H, N, d = shape.n_kv_heads, shape.tokens_per_block, shape.head_dim
    cache = torch.empty((shape.n_layers, 2, shape.blocks_per_layer, H, N, d), dtype=torch.float16, device=device)
    for l in range(shape.n_layers):
        cache[l].copy_(layer_torch(shape, l, device))
    return cache


@dataclass(frozen=True)
class GatherPattern:
    """Decode-step prefetch pattern (70B shape): per-sequence lengths, a block table that places
    each sequence's logical blocks at random slots of the per-layer pool, and k predicted logical
    block ids per sequence per step."""
    n_seq: int
    k: int
    lengths: np.ndarray       # int32 [n_seq] tokens
    n_blocks: np.ndarray      # int32 [n_seq] = ceil(len/16)
    block_table: np.ndarray   # int32 [n_seq][max_blocks], -1 beyond a sequence's blocks
    pool_blocks_per_layer: int
    seed: int

    @property
    def max_blocks(self) -> int:
        return int(self.block_table.shape[1])

    def predictions(self, step: int) -> np.ndarray:
        """int32 [n_seq][k]: logical block ids uniform over each sequence's blocks."""
        g = _rng(self.seed, TAG_PRED, step)
        r = g.random((self.n_seq, self.k))
        return np.minimum((r * self.n_blocks[:, None]).astype(np.int32), self.n_blocks[:, None] - 1).astype(np.int32)


def gather_pattern(n_seq: int = 64, k: int = 8, len_lo: int = 512, len_hi: int = 8192, tokens_per_block: int = 16,
                   seed: int = 0) -> GatherPattern:
    lengths = _rng(seed, TAG_LEN).integers(len_lo, len_hi + 1, size=n_seq).astype(np.int32)
    nb = ((lengths + tokens_per_block - 1) // tokens_per_block).astype(np.int32)
    total = int(nb.sum())
    perm = _rng(seed, TAG_PERM).permutation(total).astype(np.int32)
    table = np.full((n_seq, int(nb.max())), -1, np.int32)
    o = 0
    for s in range(n_seq):
        table[s, : nb[s]] = perm[o:o + nb[s]]
        o += int(nb[s])
    return GatherPattern(n_seq, k, lengths, nb, table, total, seed)


def gather_layer_torch(shape: KVShape, pat: GatherPattern, layer: int, device):
    """One layer of the decode-gather pool source, block-major float16 [pool_blocks][2][head][N][d]; the
    last block of every sequence is zero beyond the sequence's length."""
    x = layer_torch(shape, layer, device, block_major=True, n_blocks=pat.pool_blocks_per_layer)
    N = shape.tokens_per_block
    for s in range(pat.n_seq):
        tail = int(pat.lengths[s]) % N
        if tail:
            x[int(pat.block_table[s, pat.n_blocks[s] - 1]), :, :, tail:, :] = 0
    return x


def ar1_pages_torch(n_pages: int, device, rho: float = 0.95, outlier_channel: int = 77, d: int = 128, N: int = 16,
                    seed: int = 0):
    """Pages whose channels are correlated along the channel index (an AR(1) process with coefficient
    rho, unit variance) plus one x10 channel: float16 [n_pages][N][d].  Stands in for the "spatial
    correlation in attention heads" that Section 3.1 (v) says delta coding exploits; the LLaMA-shaped
    generator above has none."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(seed * 7919 + 17)
    z = torch.randn((n_pages, N, d), generator=gen, device=device, dtype=torch.float32)
    y = torch.empty_like(z)
    y[..., 0] = z[..., 0]
    c = (1.0 - rho * rho) ** 0.5
    for i in range(1, d):
        y[..., i] = rho * y[..., i - 1] + c * z[..., i]
    y[..., outlier_channel] *= 10.0
    return y.to(torch.float16)
