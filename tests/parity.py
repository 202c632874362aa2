"""Comparison of the HIP path with the CPU oracle (used by the GPU tests, smoke and bench).

Acceptance rule: skip masks equal bit for bit except on tiles whose block maximum lies within
1e-3 of the threshold; outputs within 2e-2 max-abs and 2e-3 mean-abs of the oracle, the oracle
being re-evaluated under the GPU's mask when in-band tiles differ (a legitimately flipped tile
changes the output)."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

from oracle import bsfa_oracle as orc

MAX_ABS = 2e-2
MEAN_ABS = 2e-3
BAND = 1e-3


def unpack_mask(words: np.ndarray, m_kv: int) -> np.ndarray:
    """[..., W] int32/uint32 -> [..., m_kv] bool (bit j%32 of word j/32)."""
    w = words.astype(np.uint32)
    bits = (w[..., :, None] >> np.arange(32, dtype=np.uint32)) & 1
    return bits.reshape(*w.shape[:-1], -1)[..., :m_kv].astype(bool)


@dataclass
class ParityReport:
    n_items: int
    max_abs: float
    mean_abs: float
    mask_mismatch: int          # tiles whose decision differs (all inside the band, else assert)
    in_band: int                # gateable tiles within the band
    bmax_err: float             # max |block max GPU - oracle| (nan if not dumped)
    skipped: int
    gateable: int


def compare(q, k, v, tau, block_m, block_n, causal, out_gpu, skip_mask_gpu=None, block_max_gpu=None,
            items=None, oracle_result=None, lse_gpu=None) -> ParityReport:
    """q, k, v: the bf16 tensors the kernel saw (any device); tau numpy/torch [Hq] or [Hq, T];
    out_gpu [B,N,Hq,d]; skip_mask_gpu [B,Hq,M_Q,W]; block_max_gpu [B,Hq,M_Q,M_KV].  N need not
    fill its last tile: M_Q and M_KV are rounded up and the rows that do not exist are left out."""
    qf, kf, vf = (t.detach().float().cpu() for t in (q, k, v))
    B, N, Hq, d = qf.shape
    mq, mkv = -(-N // block_m), -(-N // block_n)
    tau = np.asarray(tau.detach().cpu() if hasattr(tau, "detach") else tau, dtype=np.float32)
    if items is None:
        items = [(b, h, i) for b in range(B) for h in range(Hq) for i in range(mq)]
    items = np.asarray(items, dtype=np.int32).reshape(-1, 3)
    r = oracle_result if oracle_result is not None else orc.forward_items(qf, kf, vf, tau, block_m, block_n, causal, items)
    ib, ih, ii = items[:, 0], items[:, 1], items[:, 2]

    tau_item = tau[ih, np.minimum(ii, tau.shape[1] - 1)] if tau.ndim == 2 else tau[ih]
    gate = (r.cls == orc.CLS_SKIPPED) | (r.cls == orc.CLS_KEPT)
    band = gate & (np.abs(r.bmax - tau_item[:, None]) <= BAND)
    mismatch = 0
    ref = r
    if skip_mask_gpu is not None:
        m = unpack_mask(skip_mask_gpu.detach().cpu().numpy(), mkv)[ib, ih, ii]        # [n, mkv] True = skipped
        o_skip = r.cls == orc.CLS_SKIPPED
        diff = m != o_skip
        assert not (m & ~gate).any(), "GPU skipped a block that is not gateable"
        assert not (diff & ~band).any(), "skip decisions differ outside the 1e-3 band: %d tiles" % int((diff & ~band).sum())
        mismatch = int(diff.sum())
        if mismatch:
            ref = orc.forward_items(qf, kf, vf, tau, block_m, block_n, causal, items, forced_keep=(~m).astype(np.uint8))
    bmax_err = float("nan")
    if block_max_gpu is not None:
        bg = block_max_gpu.detach().cpu().numpy()[ib, ih, ii]
        assert (np.isnan(bg) == np.isnan(r.bmax)).all(), "block_max NaN pattern differs"
        bmax_err = float(np.nanmax(np.abs(bg - r.bmax))) if gate.any() else 0.0
        assert bmax_err <= 1e-4 * max(1.0, float(np.nanmax(np.abs(r.bmax))) if gate.any() else 1.0), "block maxima differ by %g" % bmax_err
    if lse_gpu is not None:
        lg = _tile_rows(lse_gpu.detach().cpu().numpy()[..., None], mq, block_m)[ib, ii, :, ih, 0]   # [n, BM]
        real = ~np.isnan(ref.lse)
        assert np.isfinite(lg[real]).all(), "non-finite log-sum-exp"
        lse_err = float(np.abs(lg - ref.lse)[real].max())
        assert lse_err <= 5e-3, "log-sum-exp differs by %g" % lse_err
    og = _tile_rows(out_gpu.detach().float().cpu().numpy(), mq, block_m)[ib, ii, :, ih]  # [n, BM, d]
    real = ~np.isnan(ref.out)                                                            # rows that exist
    assert np.isfinite(og[real]).all(), "non-finite output"
    err = np.abs(og - ref.out)[real]
    rep = ParityReport(len(items), float(err.max()), float(err.mean()), mismatch, int(band.sum()), bmax_err,
                       int((ref.cls == orc.CLS_SKIPPED).sum()), int(gate.sum()))
    assert rep.max_abs <= MAX_ABS, "max-abs error %g > %g" % (rep.max_abs, MAX_ABS)
    assert rep.mean_abs <= MEAN_ABS, "mean-abs error %g > %g" % (rep.mean_abs, MEAN_ABS)
    return rep


def _tile_rows(x: np.ndarray, mq: int, block_m: int) -> np.ndarray:
    """[B, N, H, c] -> [B, mq, block_m, H, c], the rows past N filled with NaN."""
    B, N = x.shape[:2]
    if mq * block_m != N:
        pad = np.full((B, mq * block_m - N) + x.shape[2:], np.nan, x.dtype)
        x = np.concatenate([x, pad], axis=1)
    return x.reshape(B, mq, block_m, *x.shape[2:])


def sample_items(shape, n_random=5, seed=0):
    """Stratified (b, h, i) sample: one query head per KV group (rotating the in-group index),
    tiles 0, 1, M_Q-1 and ``n_random`` random ones."""
    rng = np.random.default_rng(seed)
    items = []
    for g in range(shape.n_kv_heads):
        h = g * shape.group + (g % shape.group)
        tiles = {0, min(1, shape.m_q - 1), shape.m_q - 1}
        while len(tiles) < min(shape.m_q, 3 + n_random):
            tiles.add(int(rng.integers(0, shape.m_q)))
        items += [(0, h, i) for i in sorted(tiles)]
    return items
