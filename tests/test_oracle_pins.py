"""Pins of the CPU oracle against things other than itself: brute force on the full N x N
matrix, closed forms, invariants, special cases that reduce to a library softmax, the
step-by-step form of Algorithm 1, and the predicted densities the paper prints."""
import os

import numpy as np
import pytest
import torch

from paper_2512_07011_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---- independent brute force: materialise the N x N matrix (Section 2.1) -----------------
def brute_scores(q, k, causal=True):
    """[B,Hq,N,N] fp64 scores with the causal mask as -inf; GQA by repeating KV heads."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    G = q.shape[2] // k.shape[2]
    kk = np.repeat(k, G, axis=2)
    S = np.einsum("bnhd,bmhd->bhnm", q, kk) / np.sqrt(q.shape[-1])
    if causal:
        N = q.shape[1]
        S = np.where(np.triu(np.ones((N, N), bool), 1)[None, None], -np.inf, S)
    return S


def brute_attention(q, k, v, causal=True, key_keep=None):
    """softmax(S) V with an optional boolean [B,Hq,N,N] entry mask of kept positions."""
    S = brute_scores(q, k, causal)
    if key_keep is not None:
        S = np.where(key_keep, S, -np.inf)
    with np.errstate(invalid="ignore"):          # rows left without any key (partial key_keep masks) become NaN
        P = np.exp(S - S.max(axis=-1, keepdims=True))
        P /= P.sum(axis=-1, keepdims=True)
    G = q.shape[2] // v.shape[2]
    vv = np.repeat(np.asarray(v, np.float64), G, axis=2)
    return np.einsum("bhnm,bmhd->bnhd", P, vv), P


def block_view(S, bm, bn):
    B, H, N, _ = S.shape
    return S.reshape(B, H, N // bm, bm, N // bn, bn)


def expand_blocks(keep_blocks, bm, bn):
    """[B,H,MQ,MKV] bool -> [B,H,N,N] bool"""
    return np.repeat(np.repeat(keep_blocks, bm, axis=2), bn, axis=3)


CASES = [
    # (B, N, Hq, Hkv, d, BM, BN)
    (1, 512, 2, 2, 64, 64, 64),       # the small fp32-stated configuration: 2 heads, d=64, 64x64 tiles
    (2, 256, 4, 2, 32, 128, 64),      # the paper's tile shape, GQA 2:1, batch 2
    (1, 192, 4, 1, 16, 32, 64),       # B_M < B_N, GQA 4:1
]


def make(case, seed=0, boost=True):
    B, N, Hq, Hkv, d, BM, BN = case
    shp = synth.Shape(B, N, Hq, Hkv, d, BM, BN)
    q, k, v = synth.tiny(seed, shp, n_boost=max(1, shp.m_kv // 2) if boost else 0)
    return shp, q.numpy(), k.numpy(), v.numpy()


@pytest.mark.parametrize("case", CASES)
def test_p1_dense_equals_brute_force(oracle, case):
    shp, q, k, v = make(case)
    tau = np.full(shp.n_q_heads, -np.inf, np.float32)
    r = oracle.forward(q, k, v, tau, shp.block_m, shp.block_n)
    ref, _ = brute_attention(q, k, v)
    assert np.abs(r.out - ref).max() < 2e-6
    assert (r.cls != oracle.CLS_SKIPPED).all()
    # LSE against the brute-force log-sum-exp
    S = brute_scores(q, k)
    lse = np.log(np.exp(S - S.max(-1, keepdims=True)).sum(-1)) + S.max(-1)
    assert np.abs(r.lse - lse.transpose(0, 2, 1)).max() < 1e-5


@pytest.mark.parametrize("case", CASES)
def test_p1_noncausal_dense_equals_brute_force(oracle, case):
    shp, q, k, v = make(case)
    tau = np.full(shp.n_q_heads, -np.inf, np.float32)
    r = oracle.forward(q, k, v, tau, shp.block_m, shp.block_n, causal=False)
    ref, _ = brute_attention(q, k, v, causal=False)
    assert np.abs(r.out - ref).max() < 2e-6


@pytest.mark.parametrize("case", CASES)
def test_p2_exhaustive_skip_enumeration(oracle, case):
    """Every block maximum recomputed from the N x N matrix; every decision listed; sweeping
    tau over the sorted maxima of a head skips 0, 1, ..., n-1 tiles with nested keep-sets."""
    shp, q, k, v = make(case, seed=3)
    bm, bn = shp.block_m, shp.block_n
    S = brute_scores(q, k)
    blk = block_view(S, bm, bn)
    bmax_ref = blk.max(axis=(3, 5))                         # [B,H,MQ,MKV]
    i = np.arange(shp.m_q)[:, None]
    j = np.arange(shp.m_kv)[None, :]
    reach = j * bn <= (i + 1) * bm - 1
    # gateable <=> no entry of the tile is masked
    gate = np.isfinite(blk).all(axis=(3, 5))
    assert (gate == ((j + 1) * bn - 1 <= i * bm)[None, None]).all()
    r = oracle.forward(q, k, v, np.full(shp.n_q_heads, -np.inf, np.float32), bm, bn)
    assert ((r.cls == oracle.CLS_UNREACHABLE) == ~reach[None, None]).all()
    assert ((r.cls == oracle.CLS_DIAGONAL) == (reach & ~gate[0, 0])[None, None]).all()
    assert np.isnan(r.bmax[~gate]).all()
    np.testing.assert_allclose(r.bmax[gate], bmax_ref[gate], rtol=0, atol=1e-6)

    for h in range(shp.n_q_heads):
        vals = np.sort(r.bmax[:, h][gate[:, h]])
        assert np.unique(vals).size == vals.size            # generator gives distinct maxima
        prev_keep = None
        for n_skip, t in enumerate(list(vals) + [np.inf]):
            tau = np.full(shp.n_q_heads, -np.inf, np.float32)
            tau[h] = t
            rr = oracle.forward(q, k, v, tau, bm, bn)
            skipped = rr.cls[:, h] == oracle.CLS_SKIPPED
            assert skipped.sum() == n_skip                  # keep on equality (s_max >= tau)
            assert rr.counts[:, h, 0].sum() == n_skip
            expect = gate[:, h] & (r.bmax[:, h] < t)
            assert (skipped == expect).all()
            keep = ~skipped
            if prev_keep is not None:
                assert (keep <= prev_keep).all()            # nested
            prev_keep = keep
            # other heads untouched
            assert (rr.cls[:, [x for x in range(shp.n_q_heads) if x != h]] != oracle.CLS_SKIPPED).all()


@pytest.mark.parametrize("case", CASES)
def test_p3_p7_masked_softmax_rowsums_and_decomposition(oracle, case):
    shp, q, k, v = make(case, seed=5)
    bm, bn = shp.block_m, shp.block_n
    dense = oracle.forward(q, k, v, np.full(shp.n_q_heads, -np.inf, np.float32), bm, bn)
    tau = oracle.calibrate(dense.bmax, dense.cls, [0.5])[0]
    r = oracle.forward(q, k, v, tau, bm, bn)
    assert 0 < (r.cls == oracle.CLS_SKIPPED).sum()
    # P3: probabilities over kept blocks sum to one
    assert np.abs(r.psum - 1.0).max() < 1e-12
    # output equals brute-force attention with the skipped blocks masked out entry-wise
    keep_entries = expand_blocks(r.cls >= oracle.CLS_KEPT, bm, bn)
    ref, _ = brute_attention(q, k, v, key_keep=keep_entries)
    assert np.abs(r.out - ref).max() < 2e-6
    # P7: O_dense = (1-delta) O_kept + delta O_skipped, delta = dense mass on skipped blocks
    _, P = brute_attention(q, k, v)
    skipped_entries = expand_blocks(r.cls == oracle.CLS_SKIPPED, bm, bn)
    delta = (P * skipped_entries).sum(-1).transpose(0, 2, 1)          # [B,N,H]
    Ps = P * skipped_entries
    G = shp.group
    vv = np.repeat(np.asarray(v, np.float64), G, axis=2)
    o_sk_unnorm = np.einsum("bhnm,bmhd->bnhd", Ps, vv)                # = delta * O_skipped
    recon = (1 - delta)[..., None] * r.out + o_sk_unnorm
    assert np.abs(recon - dense.out).max() < 5e-6
    bound = 2 * delta * np.abs(v).max()
    assert (np.abs(dense.out - r.out).max(-1) <= bound + 1e-6).all()


def test_p4_tau_plus_inf_is_per_tile_causal_softmax(oracle):
    """B_M = B_N: only the diagonal block survives; inside a tile that is the textbook causal
    softmax, evaluated here with torch's library softmax."""
    shp, q, k, v = make(CASES[0], seed=7)
    bm = shp.block_m
    r = oracle.forward(q, k, v, np.full(shp.n_q_heads, np.inf, np.float32), bm, bm)
    assert ((r.cls == oracle.CLS_KEPT).sum()) == 0
    tq, tk, tv = (torch.from_numpy(x).double() for x in (q, k, v))
    for h in range(shp.n_q_heads):
        for i in range(shp.m_q):
            sl = slice(i * bm, (i + 1) * bm)
            s = tq[0, sl, h] @ tk[0, sl, h].T / np.sqrt(shp.head_dim)
            s = s.masked_fill(torch.triu(torch.ones(bm, bm, dtype=torch.bool), 1), float("-inf"))
            ref = torch.softmax(s, dim=-1) @ tv[0, sl, h]
            assert np.abs(r.out[0, sl, h] - ref.numpy()).max() < 2e-6


def test_p4_tau_plus_inf_rect_tiles(oracle):
    """128 x 64 tiles: two key blocks touch the boundary; result = attention over the tile's
    own 128 tokens."""
    shp, q, k, v = make(CASES[1], seed=8)
    r = oracle.forward(q, k, v, np.full(shp.n_q_heads, np.inf, np.float32), 128, 64)
    N = shp.seqlen
    own = (np.arange(N)[:, None] // 128) == (np.arange(N)[None, :] // 128)
    ref, _ = brute_attention(q, k, v, key_keep=own[None, None])
    assert np.abs(r.out - ref).max() < 2e-6
    assert (r.counts[..., 0] == r.counts[..., 1]).all()
    assert (r.counts[..., 2] - r.counts[..., 1] == 2 * shp.m_q).all()


@pytest.mark.parametrize("case", CASES[:2])
def test_p5_algorithm1_any_order_equals_definition(oracle, case):
    shp, q, k, v = make(case, seed=11)
    bm, bn = shp.block_m, shp.block_n
    dense = oracle.forward(q, k, v, np.full(shp.n_q_heads, -np.inf, np.float32), bm, bn)
    tau = oracle.calibrate(dense.bmax, dense.cls, [0.4])[0]
    r = oracle.forward(q, k, v, tau, bm, bn)
    rng = np.random.default_rng(0)
    for b in range(shp.batch):
        for h in range(shp.n_q_heads):
            for i in range(shp.m_q):
                gate = [j for j in range(shp.m_kv) if (j + 1) * bn - 1 <= i * bm]
                for order in (gate, gate[::-1], list(rng.permutation(gate))):
                    O, L, kept = oracle.alg1_tile(q, k, v, tau[h], b, h, i, bm, bn, order=[int(x) for x in order])
                    sl = slice(i * bm, (i + 1) * bm)
                    assert np.abs(O - r.out[b, sl, h]).max() < 2e-6
                    assert np.abs(L - r.lse[b, sl, h]).max() < 1e-5
                    assert sorted(kept) == list(np.nonzero(r.cls[b, h, i] >= oracle.CLS_KEPT)[0])


def test_p6_predicted_density_matches_paper_table(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table1_predicted_density.txt")) if not l.startswith("#")]
    assert len(rows) == 10
    for n, kk, printed in rows:
        got = oracle.predicted_density(int(n), 128, 64, int(kk))
        # the paper's samples are a little shorter than the nominal length; two printed decimals
        assert abs(got - float(printed)) <= 0.0101, (n, kk, printed, got)


def test_p6_topk_calibration_reproduces_predicted_density(oracle):
    """Thresholds = exact per-tile k-th largest block maximum on the same sample: the measured
    density counted by the oracle equals the closed form."""
    shp = synth.Shape(1, 1024, 2, 1, 16, 128, 64)
    q, k, v = synth.tiny(2, shp, n_boost=4)
    dense = oracle.forward(q, k, v, np.full(2, -np.inf, np.float32), 128, 64)
    gate = oracle.gateable_mask(1024, 128, 64)
    for kk in (1, 3, 6, 14, 20):
        T = oracle.calibrate_topk([dense.bmax[0]], gate, [kk])[0]            # [Hq, MQ]
        r = oracle.forward(q, k, v, T, 128, 64)
        kept_gate = (r.cls == oracle.CLS_KEPT).sum(-1)                         # [B,H,MQ]
        A = gate.sum(1)
        assert (kept_gate == np.minimum(kk, A)[None, None]).all()
        dens = 1 - r.counts[..., 0].sum() / r.counts[..., 2].sum()
        assert abs(dens - oracle.predicted_density(1024, 128, 64, kk)) < 1e-12


def test_tie_rule_and_uniform_closed_form(oracle):
    """Q = 0: every score is 0, every block maximum is 0.  tau = 0 keeps everything (keep on
    equality) and the output is the running mean of V; the next float above 0 skips every
    gateable block and the output is the mean over the tile's own visible tokens."""
    shp = synth.Shape(1, 256, 2, 1, 8, 64, 64)
    _, k, v = synth.tiny(4, shp, n_boost=0)
    q = np.zeros((1, 256, 2, 8), np.float32)
    v = v.numpy().astype(np.float64)
    r = oracle.forward(q, k, v, np.zeros(2, np.float32), 64, 64)
    assert (r.cls != oracle.CLS_SKIPPED).all()
    run_mean = np.cumsum(v[0, :, 0], axis=0) / np.arange(1, 257)[:, None]
    assert np.abs(r.out[0, :, 0] - run_mean).max() < 1e-6
    tiny_pos = np.full(2, np.nextafter(np.float32(0), np.float32(1)), np.float32)
    r = oracle.forward(q, k, v, tiny_pos, 64, 64)
    assert r.counts[0, 0, 0] == r.counts[0, 0, 1] == 6          # 3+2+1 gateable tiles, all skipped
    vt = v[0, :, 0].reshape(4, 64, 8)
    own_mean = np.cumsum(vt, axis=1) / np.arange(1, 65)[None, :, None]
    assert np.abs(r.out[0, :, 0] - own_mean.reshape(256, 8)).max() < 1e-6


def test_p8_p9_constant_and_indicator_values(oracle):
    shp, q, k, v = make(CASES[1], seed=13)
    bm, bn = shp.block_m, shp.block_n
    dense = oracle.forward(q, k, v, np.full(shp.n_q_heads, -np.inf, np.float32), bm, bn)
    tau = oracle.calibrate(dense.bmax, dense.cls, [0.5])[0]
    v0 = np.linspace(-1, 1, shp.head_dim).astype(np.float32)
    vc = np.broadcast_to(v0, v.shape).copy()
    r = oracle.forward(q, k, vc, tau, bm, bn)
    assert np.abs(r.out - v0).max() < 1e-6
    # indicator V: column c collects the mass on key blocks with index = c (M_KV <= d here)
    vi = np.zeros_like(v)
    for j in range(shp.m_kv):
        vi[:, j * bn:(j + 1) * bn, :, j] = 1.0
    r = oracle.forward(q, k, vi, tau, bm, bn)
    mass = r.out.reshape(shp.batch, shp.m_q, bm, shp.n_q_heads, shp.head_dim)[..., :shp.m_kv]
    skipped = (r.cls == oracle.CLS_SKIPPED).transpose(0, 2, 1, 3)[:, :, None]     # [B,MQ,1,H,MKV]
    assert (mass[np.broadcast_to(skipped, mass.shape)] == 0).all()
    assert np.abs(mass.sum(-1) - 1).max() < 1e-6


def test_p10_gqa_degeneracy(oracle):
    shp, q, k, v = make(CASES[2], seed=17)
    q[:, :, 1:] = q[:, :, :1]                                  # 4 query heads, 1 KV head
    dense = oracle.forward(q, k, v, np.full(4, -np.inf, np.float32), shp.block_m, shp.block_n)
    tau = oracle.calibrate(dense.bmax, dense.cls, [0.5])[0]
    assert np.unique(tau).size == 1
    r = oracle.forward(q, k, v, tau, shp.block_m, shp.block_n)
    for h in range(1, 4):
        assert (r.out[:, :, h] == r.out[:, :, 0]).all()
        assert (r.cls[:, h] == r.cls[:, 0]).all()
    # MHA written as GQA with repeated KV heads gives the same numbers
    k4, v4 = np.repeat(k, 4, axis=2), np.repeat(v, 4, axis=2)
    r4 = oracle.forward(q, k4, v4, tau, shp.block_m, shp.block_n)
    assert (r4.out == r.out).all()


def test_calibrate_order_statistic_and_generalisation(oracle):
    shp, q, k, v = make(CASES[0], seed=21)
    bm = shp.block_m
    dense = oracle.forward(q, k, v, np.full(2, -np.inf, np.float32), bm, bm)
    fr = [0.0, 0.25, 0.5, 0.75, 0.9, 1.0]
    taus = oracle.calibrate(dense.bmax, dense.cls, fr)
    assert np.isneginf(taus[0]).all() and np.isposinf(taus[-1]).all()
    n_gate = dense.counts[0, :, 1]
    assert (n_gate == 28).all() and (dense.counts[0, :, 2] == 36).all()
    for li, f in enumerate(fr):
        r = oracle.forward(q, k, v, taus[li], bm, bm)
        assert (r.counts[0, :, 0] == np.floor(f * n_gate)).all()
    # forced mask overrides the gate and nothing else
    forced = (dense.cls >= oracle.CLS_KEPT).astype(np.uint8)
    forced[0, 0, 5, 2] = 0
    r = oracle.forward(q, k, v, np.full(2, -np.inf, np.float32), bm, bm, forced_keep=forced)
    assert r.cls[0, 0, 5, 2] == oracle.CLS_SKIPPED and (r.cls == oracle.CLS_SKIPPED).sum() == 1


def test_items_subset_matches_full(oracle):
    shp, q, k, v = make(CASES[1], seed=23)
    dense = oracle.forward(q, k, v, np.full(4, -np.inf, np.float32), 128, 64)
    tau = oracle.calibrate(dense.bmax, dense.cls, [0.5])[0]
    full = oracle.forward(q, k, v, tau, 128, 64)
    items = [(1, 3, 1), (0, 0, 0), (0, 2, 1)]
    r = oracle.forward_items(q, k, v, tau, 128, 64, items=items)
    for n, (b, h, i) in enumerate(items):
        assert (r.out[n] == full.out[b, i * 128:(i + 1) * 128, h]).all()
        assert (r.cls[n] == full.cls[b, h, i]).all()


# ---- sequences that do not fill their last block, thresholds shorter than the sequence -------
RAGGED = [
    # (B, N_aligned, Hq, Hkv, d, BM, BN), N
    ((1, 512, 2, 2, 64, 64, 64), 450),       # partial last tile and block
    ((2, 512, 4, 2, 32, 128, 64), 322),      # last tile covers 66 of 128 rows, 3 blocks of which one partial
    ((1, 384, 4, 1, 16, 128, 64), 260),      # last tile's second boundary block is padding only
    ((1, 256, 4, 2, 16, 32, 64), 197),       # B_M < B_N
    ((1, 128, 2, 1, 16, 128, 64), 1),        # a single token
]


def ragged_reference(q, k, v, tau_tiles, bm, bn):
    """What Section 4.3's padding rule must amount to, from the real N x N matrix only: block
    maxima over the rows and columns that exist, the gate on blocks that lie entirely before
    the tile's first row, masked softmax over kept entries.  tau_tiles [Hq, MQ]."""
    B, N, Hq, d = q.shape
    MQ, MKV = -(-N // bm), -(-N // bn)
    S = brute_scores(q, k)
    keep = np.ones((B, Hq, N, N), bool)
    bmax = np.full((B, Hq, MQ, MKV), np.nan)
    skipped = np.zeros((B, Hq, MQ, MKV), bool)
    for i in range(MQ):
        r0, r1 = i * bm, min((i + 1) * bm, N)
        for j in range(MKV):
            c0, c1 = j * bn, min((j + 1) * bn, N)
            if (j + 1) * bn - 1 <= r0:                        # gateable: whole block visible to every row
                assert c1 == (j + 1) * bn
                m = S[:, :, r0:r1, c0:c1].max(axis=(2, 3))    # [B,Hq]
                bmax[:, :, i, j] = m
                sk = m.astype(np.float32) < tau_tiles[None, :, i]
                skipped[:, :, i, j] = sk
                keep[:, :, r0:r1, c0:c1] = ~sk[:, :, None, None]
    out, _ = brute_attention(q, k, v, key_keep=keep)
    return out, bmax, skipped


@pytest.mark.parametrize("case,N", RAGGED)
def test_p11_ragged_padding_equals_ignoring_out_of_range(oracle, case, N):
    shp, q, k, v = make(case, seed=31)
    q, k, v = (np.ascontiguousarray(x[:, :N]) for x in (q, k, v))
    bm, bn, Hq = shp.block_m, shp.block_n, shp.n_q_heads
    MQ, MKV = -(-N // bm), -(-N // bn)
    dense = oracle.forward(q, k, v, np.full(Hq, -np.inf, np.float32), bm, bn)
    assert dense.out.shape == q.shape and dense.bmax.shape == (shp.batch, Hq, MQ, MKV)
    ref, bmax_ref, _ = ragged_reference(q, k, v, np.full((Hq, MQ), -np.inf, np.float32), bm, bn)
    assert np.abs(dense.out - ref).max() < 2e-6
    gate = ~np.isnan(bmax_ref)
    assert (gate == np.broadcast_to(oracle.gateable_mask(N, bm, bn), gate.shape)).all()
    assert (np.isnan(dense.bmax) == ~gate).all()
    np.testing.assert_allclose(dense.bmax[gate], bmax_ref[gate], rtol=0, atol=1e-6)
    i = np.arange(MQ)[:, None]
    j = np.arange(MKV)[None, :]
    reach = j * bn <= np.minimum((i + 1) * bm, N) - 1
    assert ((dense.cls != oracle.CLS_UNREACHABLE) == reach[None, None]).all()
    if gate.any():
        # per-tile thresholds at the median of each head's maxima, shifted per tile
        med = np.array([np.median(dense.bmax[:, h][gate[:, h]]) for h in range(Hq)], np.float32)
        tau = (med[:, None] + 0.05 * np.arange(MQ)[None, :]).astype(np.float32)
        r = oracle.forward(q, k, v, tau, bm, bn)
        ref, _, skipped = ragged_reference(q, k, v, tau, bm, bn)
        assert ((r.cls == oracle.CLS_SKIPPED) == skipped).all()
        assert 0 < skipped.sum() < gate.sum()
        assert np.abs(r.out - ref).max() < 2e-6
        assert (r.counts[..., 0] == skipped.sum(axis=(2, 3))).all()
        assert (r.counts[..., 2] == reach.sum()).all()


def test_p12_thresholds_beyond_calibrated_length_reuse_last(oracle):
    """Section 4.3: positions past the calibrated length take the last calibrated thresholds."""
    shp, q, k, v = make(CASES[0], seed=37)
    bm, bn, Hq = shp.block_m, shp.block_n, shp.n_q_heads
    dense = oracle.forward(q, k, v, np.full(Hq, -np.inf, np.float32), bm, bn)
    gate = oracle.gateable_mask(shp.seqlen, bm, bn)
    T = 3
    rng = np.random.default_rng(5)
    short = (np.nanmedian(dense.bmax[0], axis=(1, 2))[:, None] + rng.normal(0, 0.3, (Hq, T))).astype(np.float32)
    r = oracle.forward(q, k, v, short, bm, bn)
    used = short[:, np.minimum(np.arange(shp.m_q), T - 1)]               # [Hq, MQ]
    expect = gate[None, None] & (dense.bmax < used[None, :, :, None])
    assert ((r.cls == oracle.CLS_SKIPPED) == expect).all() and expect.any()
    ref, _, _ = ragged_reference(q, k, v, used, bm, bn)
    assert np.abs(r.out - ref).max() < 2e-6


# ---- bidirectional gate (Section 4.3, last sentence) and top-k averaged over samples (Section 4.2) ----
@pytest.mark.parametrize("case", CASES)
def test_p13_noncausal_gate_split_and_output_from_the_full_matrix(oracle, case):
    """causal = 0 with finite thresholds: the blocks that overlap the tile's own token range are
    always kept, every other block is gated on its maximum.  Classes, maxima, kept set and
    output are recomputed here from the unmasked N x N matrix with explicit token ranges."""
    shp, q, k, v = make(case, seed=41)
    bm, bn, Hq = shp.block_m, shp.block_n, shp.n_q_heads
    S = brute_scores(q, k, causal=False)
    bmax_ref = block_view(S, bm, bn).max(axis=(3, 5))                   # [B,H,MQ,MKV]
    own = np.zeros((shp.m_q, shp.m_kv), bool)
    for i in range(shp.m_q):
        rows = set(range(i * bm, (i + 1) * bm))
        for j in range(shp.m_kv):
            own[i, j] = bool(rows & set(range(j * bn, (j + 1) * bn)))     # shares a token index with the tile
    assert own.sum(1).min() >= 1 and (~own).any()
    assert (oracle.gateable_mask(shp.seqlen, bm, bn, causal=False) == ~own).all()
    dense = oracle.forward(q, k, v, np.full(Hq, -np.inf, np.float32), bm, bn, causal=False)
    assert ((dense.cls == oracle.CLS_DIAGONAL) == own[None, None]).all()
    assert (dense.cls != oracle.CLS_UNREACHABLE).all() and (dense.cls != oracle.CLS_SKIPPED).all()
    gate = np.broadcast_to(~own, bmax_ref.shape)
    assert np.isnan(dense.bmax[~gate]).all()
    np.testing.assert_allclose(dense.bmax[gate], bmax_ref[gate], rtol=0, atol=1e-6)
    # per-head thresholds at the 40 % order statistic of the head's gateable maxima
    tau = np.array([np.sort(bmax_ref[:, h][gate[:, h]].astype(np.float32))[int(0.4 * gate[:, h].sum())]
                    for h in range(Hq)], np.float32)
    r = oracle.forward(q, k, v, tau, bm, bn, causal=False)
    skipped = gate & (bmax_ref.astype(np.float32) < tau[None, :, None, None])
    assert 0 < skipped.sum() < gate.sum()
    assert ((r.cls == oracle.CLS_SKIPPED) == skipped).all()
    assert ((r.cls == oracle.CLS_DIAGONAL) == own[None, None]).all()
    assert (r.counts[..., 0] == skipped.sum(axis=(2, 3))).all()
    assert (r.counts[..., 1] == (~own).sum()).all() and (r.counts[..., 2] == own.size).all()
    ref, _ = brute_attention(q, k, v, causal=False, key_keep=expand_blocks(~skipped, bm, bn))
    assert np.abs(r.out - ref).max() < 2e-6
    assert np.abs(r.psum - 1.0).max() < 1e-12
    # +inf keeps exactly the own-range blocks
    r = oracle.forward(q, k, v, np.full(Hq, np.inf, np.float32), bm, bn, causal=False)
    ref, _ = brute_attention(q, k, v, causal=False, key_keep=expand_blocks(np.broadcast_to(own, gate.shape), bm, bn))
    assert np.abs(r.out - ref).max() < 2e-6


def test_p14_topk_thresholds_are_the_mean_over_samples(oracle):
    """Three calibration samples: per (head, tile) the k-th largest gateable block maximum of
    each sample, taken here from the N x N matrices with a plain sort, then numpy's mean; -inf
    (tile has at most k gateable blocks) and +inf (k = 0) sit in the same places."""
    shp = synth.Shape(1, 1024, 4, 2, 16, 128, 64)
    bm, bn, Hq = 128, 64, 4
    samples, per_sample = [], []
    ks = [0, 1, 3, 5, 40]
    for seed in (51, 52, 53):
        q, k, v = synth.tiny(seed, shp, n_boost=4)
        S = brute_scores(q.numpy(), k.numpy())
        blk = block_view(S, bm, bn)
        full = np.isfinite(blk).all(axis=(3, 5))[0, 0]                # [MQ,MKV] gateable = nothing masked
        bmax = blk.max(axis=(3, 5))[0].astype(np.float32)              # [Hq,MQ,MKV]
        samples.append(np.where(full[None], bmax, np.nan))
        T = np.empty((len(ks), Hq, shp.m_q), np.float64)
        for h in range(Hq):
            for i in range(shp.m_q):
                x = np.sort(bmax[h, i][full[i]])[::-1]
                for li, kk in enumerate(ks):
                    T[li, h, i] = np.inf if kk == 0 and x.size > 0 else (-np.inf if x.size <= kk else x[kk - 1])
        per_sample.append(T)
    gate = oracle.gateable_mask(1024, bm, bn)
    assert (gate == full).all()
    got = oracle.calibrate_topk(samples, gate, ks)
    with np.errstate(invalid="ignore"):
        want = np.mean(np.stack(per_sample), axis=0)
    assert (np.isinf(got) == np.isinf(want)).all() and (np.sign(got[np.isinf(got)]) == np.sign(want[np.isinf(want)])).all()
    fin = np.isfinite(want)
    assert fin.any() and np.isinf(want).any()
    np.testing.assert_allclose(got[fin], want[fin].astype(np.float32), rtol=2e-7, atol=0)
    # the three samples differ, so the mean differs from every single-sample result
    for T in per_sample:
        assert np.abs(T[fin] - want[fin]).max() > 1e-3
    # one sample is its own mean
    one = oracle.calibrate_topk(samples[:1], gate, ks)
    f1 = np.isfinite(per_sample[0])
    np.testing.assert_array_equal(one[f1], per_sample[0][f1].astype(np.float32))


# ---- the comparison predicate of Section 3 (running-maximum filter) ---------------------------------
def test_p15_running_max_predicate_limits_and_error_bound(oracle):
    """lambda = -inf keeps everything (dense); lambda = +inf keeps nothing the gate applies to (the
    statistic is never above 0); for lambda <= 0 every skipped score lies at least |lambda| below its
    row's final maximum, so the dense softmax mass of the skipped keys is at most
    n_skipped_keys * exp(lambda) and the output moves by at most twice that times max|V|."""
    shp, q, k, v = make(CASES[1], seed=61)
    bm, bn = shp.block_m, shp.block_n
    dense, _ = brute_attention(q, k, v)
    _, P = brute_attention(q, k, v)
    N = shp.seqlen
    for b in range(shp.batch):
        for h in range(shp.n_q_heads):
            for i in range(shp.m_q):
                sl = slice(i * bm, (i + 1) * bm)
                gate = [j for j in range(shp.m_kv) if (j + 1) * bn - 1 <= i * bm]
                reach = [j for j in range(shp.m_kv) if j * bn <= (i + 1) * bm - 1]
                O, L, kept, st = oracle.alg1_tile_running_max(q, k, v, -np.inf, b, h, i, bm, bn)
                assert kept == reach and np.abs(O - dense[b, sl, h]).max() < 2e-6
                assert all(x <= 0 for x in st.values())
                O, L, kept, st = oracle.alg1_tile_running_max(q, k, v, np.inf, b, h, i, bm, bn)
                assert kept == [j for j in reach if j not in gate]
                own = np.zeros((1, 1, N, N), bool)
                for j in kept:
                    own[0, 0, sl, j * bn:(j + 1) * bn] = True
                ref, _ = brute_attention(q[b:b + 1, :, h:h + 1], k[b:b + 1, :, h // shp.group:h // shp.group + 1],
                                         v[b:b + 1, :, h // shp.group:h // shp.group + 1], key_keep=own)
                assert np.abs(O - ref[0, sl, 0]).max() < 2e-6
    # a problem on which the predicate does skip: queries share a direction and the first key block is
    # boosted along it, so the running maximum is set early and most later blocks fall far below it
    big = synth.Shape(1, 1024, 2, 1, 16, 128, 64)
    rng = np.random.default_rng(7)
    u = rng.normal(size=16); u /= np.linalg.norm(u)
    q = (3.0 * u + 0.4 * rng.normal(size=(1, 1024, 2, 16))).astype(np.float32)
    k = rng.normal(size=(1, 1024, 1, 16)).astype(np.float32)
    k[:, :64] += (4.0 * u).astype(np.float32)
    v = rng.normal(size=(1, 1024, 1, 16)).astype(np.float32)
    dense, P = brute_attention(q, k, v)
    N, skipped_any, kept_any = 1024, 0, 0
    for lam in (-0.5, -2.0, -6.0):
        for h in range(2):
            for i in (3, 7):
                sl = slice(i * bm, (i + 1) * bm)
                O, L, kept, st = oracle.alg1_tile_running_max(q, k, v, lam, 0, h, i, bm, bn)
                skipped = [j for j in st if j not in kept]
                skipped_any += len(skipped)
                kept_any += len([j for j in st if j in kept and j > 0])
                delta = np.zeros(bm)
                for j in skipped:
                    delta += P[0, h, sl, j * bn:(j + 1) * bn].sum(-1)
                assert (delta <= len(skipped) * bn * np.exp(lam) + 1e-12).all()
                assert (np.abs(O - dense[0, sl, h]).max(-1) <= 2 * delta * np.abs(v).max() + 1e-6).all()
                # the kept set reproduces the output: exact softmax over the kept blocks
                keep = np.zeros((1, 1, N, N), bool)
                for j in kept:
                    keep[0, 0, sl, j * bn:(j + 1) * bn] = True
                ref, _ = brute_attention(q[:1, :, h:h + 1], k, v, key_keep=keep)
                assert np.abs(O - ref[0, sl, 0]).max() < 2e-6
    assert skipped_any > 10 and kept_any > 0


def test_p16_running_max_predicate_closed_form(oracle):
    """All queries equal e, all keys of block j equal a_j e: every score of block j is a_j |e|^2 / sqrt(d).
    Decreasing a_j: the running maximum stays at block 0's value and block j is kept iff
    (a_j - a_0) |e|^2 / sqrt(d) >= lambda.  Increasing a_j: every block raises the maximum, the statistic
    is 0 and everything is kept for any lambda <= 0."""
    d, bm, bn, N = 16, 128, 64, 1024
    e = np.ones(d) / 2.0
    c = (e @ e) / np.sqrt(d)                                  # score per unit of a_j
    q = np.broadcast_to(e, (1, N, 1, d)).astype(np.float32).copy()
    rng = np.random.default_rng(3)
    v = rng.normal(size=(1, N, 1, d)).astype(np.float32)
    i = N // bm - 1
    gate = [j for j in range(N // bn) if (j + 1) * bn - 1 <= i * bm]
    a_dec = np.linspace(4.0, -4.0, N // bn)
    k = (np.repeat(a_dec, bn)[None, :, None, None] * e[None, None, None, :]).astype(np.float32)
    lam = -3.0
    O, L, kept, st = oracle.alg1_tile_running_max(q, k, v, lam, 0, 0, i, bm, bn)
    expect = [j for j in gate if np.float32((a_dec[j] - a_dec[0]) * c) >= np.float32(lam)]
    assert 1 < len(expect) < len(gate)
    assert [j for j in kept if j in gate] == expect
    for j in gate[1:]:
        assert abs(st[j] - (a_dec[j] - a_dec[0]) * c) < 1e-5
    a_inc = a_dec[::-1].copy()
    k = (np.repeat(a_inc, bn)[None, :, None, None] * e[None, None, None, :]).astype(np.float32)
    O, L, kept, st = oracle.alg1_tile_running_max(q, k, v, lam, 0, 0, i, bm, bn)
    assert [j for j in kept if j in gate] == gate and all(x == 0 for x in st.values())
