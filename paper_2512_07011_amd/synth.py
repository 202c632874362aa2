"""Seeded synthetic Q/K/V generators shared by the CPU oracle tests and the HIP path.

This module holds input recipes only: random draws, a few additive edits that give the
score matrix the structure the paper describes for real prompts (an attention sink at the
first positions, a handful of heavy-hitter "needle" key blocks per query tile, low scores
elsewhere: Section 2.3 and the needle-in-a-haystack discussion in Section 5), and dtype
rounding.  It contains none of the method's arithmetic (no scores, no block maxima, no
softmax) and imports neither the oracle nor the HIP binding.

Layout of every tensor: ``[B, N, H, d]`` (token-major, what a projection GEMM emits),
contiguous, last dimension the head dimension.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Shape:
    """Problem shape in the paper's notation (Section 2.2): N tokens, head dim d,
    query tiles of B_M rows and key/value blocks of B_N rows."""

    batch: int
    seqlen: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    block_m: int
    block_n: int

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def m_q(self) -> int:
        return self.seqlen // self.block_m

    @property
    def m_kv(self) -> int:
        return self.seqlen // self.block_n


TINY = Shape(batch=1, seqlen=512, n_q_heads=2, n_kv_heads=2, head_dim=64, block_m=64, block_n=64)


def llama_shape(seqlen: int, block_m: int = 128, block_n: int = 64) -> Shape:
    """One Llama-3.1-8B attention layer (32 query heads, 8 KV heads, d=128; Section 2.1
    gives d_model=4096, d=128, H=32) with the paper's tile shape (Section 5.1)."""
    return Shape(1, seqlen, 32, 8, 128, block_m, block_n)


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def n_gateable(i: int, block_m: int, block_n: int) -> int:
    """Number of key blocks that lie entirely at or before the first row of query tile i,
    i.e. blocks that need no causal masking for any row of the tile."""
    return (i * block_m + 1) // block_n


def tiny(seed: int, shape: Shape = TINY, n_boost: int = 4, boost: float = 3.0):
    """Small fp32 case: Q, K, V ~ N(0,1); per KV head, ``n_boost`` key blocks chosen
    uniformly without replacement get ``boost * u`` added to every key row, where u is the
    unit vector along the mean query row of the first query head that reads that KV head.
    Returns CPU fp32 tensors (q, k, v)."""
    s = shape
    g = _gen(seed, "cpu")
    q = torch.randn(s.batch, s.seqlen, s.n_q_heads, s.head_dim, generator=g, dtype=torch.float32)
    k = torch.randn(s.batch, s.seqlen, s.n_kv_heads, s.head_dim, generator=g, dtype=torch.float32)
    v = torch.randn(s.batch, s.seqlen, s.n_kv_heads, s.head_dim, generator=g, dtype=torch.float32)
    for b in range(s.batch):
        for kvh in range(s.n_kv_heads):
            u = q[b, :, kvh * s.group, :].mean(dim=0)
            u = u / u.norm()
            blocks = torch.randperm(s.m_kv, generator=g)[:n_boost]
            for j in blocks.tolist():
                k[b, j * s.block_n:(j + 1) * s.block_n, kvh, :] += boost * u
    return q, k, v


def llama_layer(seed: int, shape: Shape, device="cpu", dtype=torch.bfloat16,
                sink_tokens: int = 64, sink_gain: float = 4.0, n_needles: int = 8,
                q_gain: float = 1.0):
    """Long-context case: Q, K, V ~ N(0,1) (Q optionally multiplied by ``q_gain`` to sharpen
    the softmax), then, in fp32 and before rounding to ``dtype``:

    * sink: the first ``sink_tokens`` keys of every KV head get ``sink_gain * u_g`` added,
      u_g a seeded unit vector per KV head;
    * needles: for every query head h and query tile i >= 1, up to ``n_needles`` distinct
      gateable key blocks (one per equal-width stratum of the gateable range, so they are
      distinct) each get ``sqrt(d) * mhat`` added to one random key row, mhat the unit
      vector along the mean query row of tile i of head h.

    Returns (q, k, v) on ``device`` in ``dtype``."""
    s = shape
    g = _gen(seed, device)
    f32 = torch.float32
    q = torch.randn(s.batch, s.seqlen, s.n_q_heads, s.head_dim, generator=g, dtype=f32, device=device)
    if q_gain != 1.0:
        q *= q_gain
    k = torch.randn(s.batch, s.seqlen, s.n_kv_heads, s.head_dim, generator=g, dtype=f32, device=device)
    v = torch.randn(s.batch, s.seqlen, s.n_kv_heads, s.head_dim, generator=g, dtype=f32, device=device)

    # attention sink
    u = torch.randn(s.batch, s.n_kv_heads, s.head_dim, generator=g, dtype=f32, device=device)
    u = u / u.norm(dim=-1, keepdim=True)
    st = min(sink_tokens, s.seqlen)
    k[:, :st] += sink_gain * u[:, None]

    # needles
    if n_needles > 0 and s.m_q > 1:
        tiles = torch.arange(1, s.m_q, device=device)
        avail = (tiles * s.block_m + 1) // s.block_n                      # gateable blocks per tile
        # mean query row per (b, tile, head), normalised
        qm = q.view(s.batch, s.m_q, s.block_m, s.n_q_heads, s.head_dim).mean(dim=2)[:, 1:]
        mhat = qm / qm.norm(dim=-1, keepdim=True)                          # [B, MQ-1, Hq, d]
        r_blk = torch.rand(s.batch, s.m_q - 1, s.n_q_heads, n_needles, generator=g, dtype=torch.float64, device=device)
        r_row = torch.randint(0, s.block_n, (s.batch, s.m_q - 1, s.n_q_heads, n_needles), generator=g, device=device)
        n_use = torch.clamp(avail, max=n_needles)                          # [MQ-1]
        slot = torch.arange(n_needles, device=device)
        # stratum s of n_use equal strata of [0, avail): block = floor((s + r) * avail / n_use)
        blk = torch.floor((slot[None, None, None, :] + r_blk) * (avail / n_use)[None, :, None, None]).long()
        blk = torch.minimum(blk, (avail - 1)[None, :, None, None])
        valid = (slot[None, None, None, :] < n_use[None, :, None, None]).expand_as(blk)
        rows = blk * s.block_n + r_row                                     # key token index
        kvh = (torch.arange(s.n_q_heads, device=device) // s.group)[None, None, :, None].expand_as(rows)
        bidx = torch.arange(s.batch, device=device)[:, None, None, None].expand_as(rows)
        flat = (bidx * s.seqlen + rows) * s.n_kv_heads + kvh               # row of k.view(-1, d)
        add = (math.sqrt(s.head_dim) * mhat)[:, :, :, None, :].expand(-1, -1, -1, n_needles, -1)
        k.view(-1, s.head_dim).index_add_(0, flat[valid], add[valid])
    return q.to(dtype), k.to(dtype), v.to(dtype)
