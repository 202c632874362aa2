"""Sequences that do not fill their last tile or block (Section 4.3: padding by repeating the
last token), per-tile thresholds shorter than the sequence (Section 4.3: reuse beyond the
calibrated length) and batches whose elements have different lengths — HIP path against the
CPU oracle through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2512_07011_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda"
SENTINEL = 7.0


def guarded(t, n):
    """bf16 GPU copy of t[:, :n] living at the start of a larger buffer whose later rows are NaN:
    a read past token n-1 poisons the result (returns the [:, :n] view)."""
    full = t.to(torch.bfloat16).to(DEV).clone()
    full[:, n:] = float("nan")
    return full[:, :n]


def run(q, k, v, tau, bm, bn, n_alloc, seqlens=None):
    """Forward into an output buffer with sentinel rows behind the sequence."""
    B, N, Hq, d = q.shape
    out_full = torch.full((B, n_alloc, Hq, d), SENTINEL, dtype=torch.bfloat16, device=DEV)
    lse_full = torch.full((B, n_alloc, Hq), SENTINEL, dtype=torch.float32, device=DEV)
    st = binding.alloc_stats(q, bm, bn, counts=True, skip_mask=True, block_max=True)
    st.lse = lse_full if N == n_alloc else None      # [B, N, Hq] must be contiguous
    out = binding.bsfa_forward(q, k, v, tau, out=out_full[:, :N], skip_stats=st, block_m=bm, block_n=bn, seqlens=seqlens)
    torch.cuda.synchronize()
    assert (out_full[:, N:] == SENTINEL).all(), "rows behind the sequence were written"
    return out, st


RAGGED = [
    # (B, N_alloc, Hq, Hkv, d, BM, BN), N
    ((1, 512, 4, 2, 128, 128, 64), 450),
    ((2, 640, 4, 2, 128, 128, 64), 577),      # one row in the last key block
    ((1, 384, 4, 1, 128, 128, 64), 260),      # the last tile's second boundary block is padding only
    ((1, 320, 2, 2, 64, 32, 64), 197),        # B_M < B_N
    ((2, 384, 4, 2, 64, 64, 64), 321),
    ((1, 128, 2, 1, 128, 128, 64), 1),        # a single token
    ((1, 1152, 16, 8, 128, 128, 64), 1100),   # 8 (batch, KV head) pairs
    ((1, 512, 3, 1, 128, 128, 64), 450),      # odd GQA group: one head per workgroup
    ((1, 512, 2, 2, 64, 128, 64), 449),
]


@pytest.mark.parametrize("case,N", RAGGED)
def test_ragged_sequence_lengths(oracle, case, N):
    shp = synth.Shape(*case)
    q, k, v = synth.tiny(sum(case) + N, shp, n_boost=max(1, shp.m_kv // 3))
    qd, kd, vd = (guarded(t, N) for t in (q, k, v))
    bm, bn = shp.block_m, shp.block_n
    neg = torch.full((shp.n_q_heads,), float("-inf"), device=DEV)
    out, st = run(qd, kd, vd, neg, bm, bn, shp.seqlen)
    rep = parity.compare(qd, kd, vd, neg, bm, bn, True, out, st.skip_mask, st.block_max)
    assert rep.skipped == 0
    dense = oracle.forward(qd.float().cpu(), kd.float().cpu(), vd.float().cpu(), neg.cpu().numpy(), bm, bn)
    assert (st.counts.cpu().numpy() == dense.counts).all()
    if rep.gateable:
        tau = oracle.calibrate(dense.bmax, dense.cls, [0.5])[0]
        out, st = run(qd, kd, vd, torch.from_numpy(tau).to(DEV), bm, bn, shp.seqlen)
        rep = parity.compare(qd, kd, vd, tau, bm, bn, True, out, st.skip_mask, st.block_max)
        assert rep.skipped > 0
        assert st.counts.cpu().numpy()[..., 0].sum() == rep.skipped


def test_ragged_lse_and_calibration(oracle):
    """Log-sum-exp rows of a partial last tile, and both calibration entry points on a sequence
    that does not fill its last block."""
    shp = synth.Shape(1, 1024, 4, 2, 128, 128, 64)
    N = 901
    q, k, v = synth.tiny(77, shp, n_boost=5)
    qd, kd, vd = (t.to(torch.bfloat16).to(DEV)[:, :N].contiguous() for t in (q, k, v))
    neg = np.full(4, -np.inf, np.float32)
    dense = oracle.forward(qd.float().cpu(), kd.float().cpu(), vd.float().cpu(), neg, 128, 64)
    taus = binding.bsfa_calibrate(qd, kd, [0.3, 0.6])
    ref = oracle.calibrate(dense.bmax, dense.cls, [0.3, 0.6])
    assert np.abs(taus.numpy() - ref).max() <= 1e-4 * np.abs(ref).max()
    T = binding.bsfa_calibrate_topk([(qd, kd)], [2, 5])
    assert tuple(T.shape) == (2, 4, 8)
    Tref = oracle.calibrate_topk([dense.bmax[0]], oracle.gateable_mask(N, 128, 64), [2, 5])
    assert (np.isinf(Tref) == np.isinf(T.numpy())).all()
    fin = np.isfinite(Tref)
    assert np.abs(T.numpy()[fin] - Tref[fin]).max() <= 1e-4 * np.abs(Tref[fin]).max()
    st = binding.alloc_stats(qd, 128, 64, skip_mask=True, block_max=True, lse=True)
    out = binding.bsfa_forward(qd, kd, vd, T[1].contiguous().to(DEV), skip_stats=st)
    torch.cuda.synchronize()
    rep = parity.compare(qd, kd, vd, T[1].numpy(), 128, 64, True, out, st.skip_mask, st.block_max, lse_gpu=st.lse)
    assert rep.skipped > 0


def test_thresholds_shorter_than_the_sequence(oracle):
    """Per-tile thresholds calibrated for 3 query tiles used on a sequence of 8 (and thresholds
    calibrated for 8 tiles used on a sequence of 5): tiles past the calibrated length take the
    last calibrated tile's threshold."""
    shp = synth.Shape(1, 1024, 4, 2, 128, 128, 64)
    q, k, v = synth.tiny(41, shp, n_boost=5)
    qd, kd, vd = (t.to(torch.bfloat16).to(DEV) for t in (q, k, v))
    neg = np.full(4, -np.inf, np.float32)
    dense = oracle.forward(qd.float().cpu(), kd.float().cpu(), vd.float().cpu(), neg, 128, 64)
    med = np.nanmedian(dense.bmax[0], axis=(1, 2)).astype(np.float32)
    short = np.ascontiguousarray(med[:, None] + np.array([0.3, -0.2, 0.05], np.float32)[None, :])
    st = binding.alloc_stats(qd, 128, 64, skip_mask=True, block_max=True)
    out = binding.bsfa_forward(qd, kd, vd, torch.from_numpy(short).to(DEV), skip_stats=st)
    torch.cuda.synchronize()
    rep = parity.compare(qd, kd, vd, short, 128, 64, True, out, st.skip_mask, st.block_max)
    assert rep.skipped > 0
    m = parity.unpack_mask(st.skip_mask.cpu().numpy(), shp.m_kv)[0]                    # [Hq, MQ, MKV]
    gate = oracle.gateable_mask(1024, 128, 64)
    used = short[:, np.minimum(np.arange(8), 2)]
    expect = gate[None] & (dense.bmax[0] < used[:, :, None])
    assert (m != expect).sum() <= rep.mask_mismatch
    # the other direction: more calibrated tiles than the sequence has
    long_T = np.ascontiguousarray(med[:, None] + 0.05 * np.arange(8, dtype=np.float32)[None, :])
    q5, k5, v5 = (t[:, :640].contiguous() for t in (qd, kd, vd))
    st = binding.alloc_stats(q5, 128, 64, skip_mask=True, block_max=True)
    out = binding.bsfa_forward(q5, k5, v5, torch.from_numpy(long_T).to(DEV), skip_stats=st)
    torch.cuda.synchronize()
    parity.compare(q5, k5, v5, long_T, 128, 64, True, out, st.skip_mask, st.block_max)


def test_batch_of_different_lengths(oracle):
    """Four sequences of 512, 130, 321 and 0 tokens in [4, 512] slots (8 batch x KV-head pairs):
    every element equals the oracle on a batch-of-one problem of its own length; nothing behind a
    sequence's end is written."""
    shp = synth.Shape(4, 512, 4, 2, 128, 128, 64)
    lens = [512, 130, 321, 0]
    q, k, v = synth.tiny(55, shp, n_boost=3)
    qd, kd, vd = (t.to(torch.bfloat16).to(DEV).clone() for t in (q, k, v))
    for b, n in enumerate(lens):
        for t in (qd, kd, vd):
            t[b, n:] = float("nan")
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    neg = np.full(4, -np.inf, np.float32)
    bmaxes = []
    for b, n in enumerate(lens):
        if n:
            d = oracle.forward(qd[b:b + 1, :n].float().cpu(), kd[b:b + 1, :n].float().cpu(), vd[b:b + 1, :n].float().cpu(), neg, 128, 64)
            bmaxes.append(d.bmax[~np.isnan(d.bmax)])
    tau = np.full(4, np.median(np.concatenate(bmaxes)), np.float32)
    out, st = run(qd, kd, vd, torch.from_numpy(tau).to(DEV), 128, 64, 512, seqlens=sl)
    counts = st.counts.cpu().numpy()
    for b, n in enumerate(lens):
        assert (out[b, n:] == SENTINEL).all() and (st.lse[b, n:] == SENTINEL).all(), "rows behind element %d's end were written" % b
        mq_b, mkv_b = -(-n // 128), -(-n // 64)
        assert torch.isnan(st.block_max[b, :, mq_b:]).all() and (st.skip_mask[b, :, mq_b:] == 0).all()
        if n == 0:
            assert (counts[b] == 0).all()
            continue
        qb, kb, vb = (t[b:b + 1, :n] for t in (qd, kd, vd))
        rep = parity.compare(qb, kb, vb, tau, 128, 64, True, out[b:b + 1, :n],
                             st.skip_mask[b:b + 1, :, :mq_b], st.block_max[b:b + 1, :, :mq_b, :mkv_b], lse_gpu=st.lse[b:b + 1, :n])
        assert torch.isnan(st.block_max[b, :, :mq_b, mkv_b:]).all()
        ref = oracle.forward(qb.float().cpu(), kb.float().cpu(), vb.float().cpu(), tau, 128, 64)
        assert np.abs(counts[b] - ref.counts[0]).max() <= rep.mask_mismatch
    assert counts[:3, :, 0].sum() > 0
    # per-head calibration pools the gateable tiles of all elements
    taus = binding.bsfa_calibrate(qd, kd, [0.5], seqlens=sl)
    pooled = np.full((4, 4, 4, 8), np.nan, np.float32)
    for b, n in enumerate(lens):
        if n:
            d = oracle.forward(qd[b:b + 1, :n].float().cpu(), kd[b:b + 1, :n].float().cpu(), vd[b:b + 1, :n].float().cpu(), neg, 128, 64)
            pooled[b, :, :d.bmax.shape[2], :d.bmax.shape[3]] = d.bmax[0]
    ref = oracle.calibrate(pooled, ~np.isnan(pooled), [0.5])
    assert np.abs(taus.numpy() - ref).max() <= 1e-4 * np.abs(ref).max()
