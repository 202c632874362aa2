"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element, on the
same seeded inputs."""
import numpy as np
import pytest
import torch

from paper_2512_07011_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda"


def run_gpu(q, k, v, tau, bm, bn, causal=True, dump=True):
    st = binding.alloc_stats(q, bm, bn, counts=True, skip_mask=True, block_max=dump, lse=dump)
    out = binding.bsfa_forward(q, k, v, tau, causal=causal, skip_stats=st, block_m=bm, block_n=bn)
    torch.cuda.synchronize()
    return out, st


def to_dev(*ts):
    return [t.to(torch.bfloat16).to(DEV) for t in ts]


def full_case(shp, q, k, v, fraction, causal=True, oracle=None):
    """Dense and gated parity on the whole problem; thresholds from the oracle's calibration of
    the same inputs so a known number of tiles is skipped."""
    qd, kd, vd = to_dev(q, k, v)
    neg = torch.full((shp.n_q_heads,), float("-inf"), device=DEV)
    out, st = run_gpu(qd, kd, vd, neg, shp.block_m, shp.block_n, causal)
    rep = parity.compare(qd, kd, vd, neg, shp.block_m, shp.block_n, causal, out, st.skip_mask, st.block_max, lse_gpu=st.lse)
    assert rep.skipped == 0 and rep.mask_mismatch == 0
    assert (st.counts[..., 0] == 0).all()
    # thresholds at the requested quantile of the oracle's block maxima
    dense = oracle.forward(qd.float().cpu(), kd.float().cpu(), vd.float().cpu(), neg.cpu().numpy(),
                           shp.block_m, shp.block_n, causal)
    assert (st.counts.cpu().numpy()[..., 1:] == dense.counts[..., 1:]).all()
    tau = oracle.calibrate(dense.bmax, dense.cls, [fraction])[0]
    taud = torch.from_numpy(tau).to(DEV)
    out, st = run_gpu(qd, kd, vd, taud, shp.block_m, shp.block_n, causal)
    rep = parity.compare(qd, kd, vd, tau, shp.block_m, shp.block_n, causal, out, st.skip_mask, st.block_max, lse_gpu=st.lse)
    assert rep.skipped > 0
    c = st.counts.cpu().numpy()
    m = parity.unpack_mask(st.skip_mask.cpu().numpy(), shp.m_kv)
    assert (c[..., 0] == m.sum(axis=(-2, -1))).all()
    return rep


def test_config1_tiny(oracle):
    """B=1, 2 heads, d=64, N=512, 64x64 tiles, boosted key blocks; inputs rounded to bf16 once
    and given to both sides; tau = -inf and the 50th percentile."""
    q, k, v = synth.tiny(0)
    rep = full_case(synth.TINY, q, k, v, 0.5, oracle=oracle)
    assert rep.gateable == 56 and rep.skipped + rep.mask_mismatch >= 26


SHAPES = [
    # B, N, Hq, Hkv, d, BM, BN
    (1, 512, 4, 2, 128, 128, 64),
    (2, 384, 4, 1, 128, 64, 64),
    (1, 320, 2, 2, 128, 32, 64),
    (2, 640, 4, 2, 64, 128, 64),
    (1, 256, 2, 1, 64, 32, 64),
    (1, 1152, 16, 8, 128, 128, 64),    # 8 (batch, KV head) pairs: the XCD-affine work mapping
    (3, 384, 12, 4, 64, 64, 64),       # 12 pairs, not a multiple of 8
]


@pytest.mark.parametrize("case", SHAPES)
@pytest.mark.parametrize("causal", [True, False])
def test_shapes(oracle, case, causal):
    shp = synth.Shape(*case)
    q, k, v = synth.tiny(sum(case), shp, n_boost=max(1, shp.m_kv // 3))
    full_case(shp, q, k, v, 0.5, causal=causal, oracle=oracle)


def test_sharp_softmax_and_llama_recipe(oracle):
    """Llama-shaped recipe at 2K with Q scaled x3 (a peaked softmax makes the output test bite)."""
    shp = synth.llama_shape(2048)
    q, k, v = synth.llama_layer(7, shp, q_gain=3.0)
    qd, kd, vd = to_dev(q, k, v)
    items = parity.sample_items(shp, n_random=3, seed=1)
    tau = binding.bsfa_calibrate(qd, kd, [0.5])[0]
    out, st = run_gpu(qd, kd, vd, tau.to(DEV), 128, 64)
    rep = parity.compare(qd, kd, vd, tau, 128, 64, True, out, st.skip_mask, st.block_max, items=items)
    assert rep.skipped > 0


def test_strided_bhnd_layout(oracle):
    """[B,H,N,d] storage viewed as [B,N,H,d]: strides, not contiguity, define the layout."""
    shp = synth.Shape(2, 256, 4, 2, 128, 128, 64)
    q, k, v = synth.tiny(5, shp)
    qd, kd, vd = [t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in to_dev(q, k, v)]
    assert not qd.is_contiguous()
    out = torch.empty(2, 4, 256, 128, dtype=torch.bfloat16, device=DEV).permute(0, 2, 1, 3)
    neg = torch.full((4,), float("-inf"), device=DEV)
    st = binding.alloc_stats(qd, 128, 64, skip_mask=True)
    binding.bsfa_forward(qd, kd, vd, neg, out=out, skip_stats=st)
    torch.cuda.synchronize()
    parity.compare(qd, kd, vd, neg, 128, 64, True, out, st.skip_mask)


def test_per_tile_thresholds(oracle):
    """Thresholds indexed by query tile (Section 4.2's T_{l,h,i}): exact per-tile top-k."""
    shp = synth.Shape(1, 1024, 4, 2, 128, 128, 64)
    q, k, v = synth.tiny(9, shp, n_boost=5)
    qd, kd, vd = to_dev(q, k, v)
    neg = np.full(4, -np.inf, np.float32)
    dense = oracle.forward(qd.float().cpu(), kd.float().cpu(), vd.float().cpu(), neg, 128, 64)
    gate = oracle.gateable_mask(1024, 128, 64)
    T = oracle.calibrate_topk([dense.bmax[0]], gate, [3])[0]                   # [Hq, MQ]
    Td = torch.from_numpy(T).to(DEV)
    out, st = run_gpu(qd, kd, vd, Td, 128, 64)
    rep = parity.compare(qd, kd, vd, T, 128, 64, True, out, st.skip_mask, st.block_max)
    kept = (~parity.unpack_mask(st.skip_mask.cpu().numpy(), shp.m_kv)) & gate[None, None]
    # top-3 per tile, up to in-band flips
    assert np.abs(kept.sum(-1) - np.minimum(3, gate.sum(1))[None, None]).sum() <= rep.mask_mismatch


def test_plus_inf_keeps_only_boundary_blocks(oracle):
    shp = synth.Shape(1, 512, 2, 2, 128, 128, 64)
    q, k, v = synth.tiny(11, shp)
    qd, kd, vd = to_dev(q, k, v)
    inf = torch.full((2,), float("inf"), device=DEV)
    out, st = run_gpu(qd, kd, vd, inf, 128, 64)
    parity.compare(qd, kd, vd, inf, 128, 64, True, out, st.skip_mask, st.block_max)
    c = st.counts.cpu().numpy()
    assert (c[..., 0] == c[..., 1]).all() and (c[..., 2] - c[..., 1] == 2 * shp.m_q).all()


def test_calibrate_matches_oracle_rule_and_generalises(oracle):
    shp = synth.llama_shape(4096)
    q, k, v = synth.llama_layer(21, shp)
    qd, kd, vd = to_dev(q, k, v)
    fr = [0.0, 0.25, 0.5, 0.75, 0.9, 1.0]
    taus = binding.bsfa_calibrate(qd, kd, fr)
    assert torch.isneginf(taus[0]).all() and torch.isposinf(taus[-1]).all()
    # the same order statistics from the kernel's own block-max dump, selected by the oracle's rule
    neg = torch.full((32,), float("-inf"), device=DEV)
    _, st = run_gpu(qd, kd, vd, neg, 128, 64)
    bm = st.block_max.cpu().numpy()
    ref = oracle.calibrate(bm, ~np.isnan(bm), fr)
    assert (ref == taus.numpy()).all()
    # exactly floor(f n) tiles skipped on the calibration sample itself
    n = st.counts.cpu().numpy()[0, :, 1]
    for li in (1, 2, 3, 4):
        _, s2 = run_gpu(qd, kd, vd, taus[li].to(DEV), 128, 64, dump=False)
        assert (s2.counts.cpu().numpy()[0, :, 0] == np.floor(np.float32(fr[li]) * n)).all()
    # held-out seed: measured skip fraction tracks the target (Section 5.2, Robustness paragraph and Table 1: within +-0.05)
    q2, k2, v2 = to_dev(*synth.llama_layer(22, shp))
    _, s3 = run_gpu(q2, k2, v2, taus[2].to(DEV), 128, 64, dump=False)
    c = s3.counts.cpu().numpy()[0]
    assert abs(c[:, 0].sum() / c[:, 1].sum() - 0.5) < 0.05


def test_gqa_degeneracy_on_gpu():
    shp = synth.Shape(1, 512, 4, 1, 128, 128, 64)
    q, k, v = synth.tiny(13, shp)
    q[:, :, 1:] = q[:, :, :1]
    qd, kd, vd = to_dev(q, k, v)
    tau = binding.bsfa_calibrate(qd, kd, [0.5])[0]
    assert tau.unique().numel() == 1
    out, st = run_gpu(qd, kd, vd, tau.to(DEV), 128, 64)
    for h in range(1, 4):
        assert torch.equal(out[:, :, h], out[:, :, 0])
        assert torch.equal(st.skip_mask[:, h], st.skip_mask[:, 0])


def test_calibrate_topk_matches_section_4_2_rule(oracle):
    """bsfa_calibrate_topk against the oracle's per-tile top-k rule applied to the kernel's own
    block-maximum dump (two calibration samples, three sparsity levels), then the thresholds in use:
    on a calibration sample every tile keeps min(k, A) gateable blocks up to in-band flips and the
    measured density equals the closed form of the paper's Metrics paragraph."""
    shp = synth.Shape(1, 2048, 4, 2, 128, 128, 64)
    samples = [to_dev(*synth.llama_layer(s, shp)) for s in (31, 32)]
    ks = [2, 8, 20]
    T = binding.bsfa_calibrate_topk([(q, k) for q, k, _ in samples], ks)          # [levels, Hq, MQ]
    gate = oracle.gateable_mask(2048, 128, 64)
    neg = torch.full((4,), float("-inf"), device=DEV)
    dumps = []
    for q, k, v in samples:
        _, st = run_gpu(q, k, v, neg, 128, 64)
        dumps.append(st.block_max.cpu().numpy()[0])
    ref = oracle.calibrate_topk(dumps, gate, ks)
    assert (np.isinf(ref) == np.isinf(T.numpy())).all()
    fin = np.isfinite(ref)
    assert np.abs(ref[fin] - T.numpy()[fin]).max() <= 1e-6 * np.abs(ref[fin]).max()
    # single-sample thresholds are exact order statistics of that sample
    T0 = binding.bsfa_calibrate_topk([samples[0][:2]], ks)
    assert (T0.numpy() == oracle.calibrate_topk(dumps[:1], gate, ks)).all()
    q, k, v = samples[0]
    for li, kk in enumerate(ks):
        out, st = run_gpu(q, k, v, T0[li].contiguous().to(DEV), 128, 64)
        rep = parity.compare(q, k, v, T0[li].numpy(), 128, 64, True, out, st.skip_mask, st.block_max, lse_gpu=st.lse)
        kept = (~parity.unpack_mask(st.skip_mask.cpu().numpy(), shp.m_kv)) & gate[None, None]
        assert np.abs(kept.sum(-1) - np.minimum(kk, gate.sum(1))[None, None]).sum() <= rep.mask_mismatch
        c = st.counts.cpu().numpy()
        dens = 1 - c[..., 0].sum() / c[..., 2].sum()
        assert abs(dens - oracle.predicted_density(2048, 128, 64, kk)) <= (rep.mask_mismatch + 0.5) / c[..., 2].sum()


F16_SHAPES = [
    (1, 512, 4, 2, 128, 128, 64),
    (2, 384, 4, 1, 64, 64, 64),
    (1, 320, 3, 1, 128, 32, 64),
    (1, 1152, 16, 8, 128, 128, 64),
]


@pytest.mark.parametrize("case", F16_SHAPES)
def test_fp16_inputs(oracle, case):
    """fp16 Q/K/V/O (the precision of the paper's kernel, Section 5.1): same path, same tolerances;
    both sides get the fp16-rounded values.  Dense, gated, and a sequence with a partial last block."""
    shp = synth.Shape(*case)
    q, k, v = synth.tiny(sum(case) + 1, shp, n_boost=max(1, shp.m_kv // 3))
    qd, kd, vd = (t.to(torch.float16).to(DEV) for t in (q, k, v))
    bm, bn = shp.block_m, shp.block_n
    neg = torch.full((shp.n_q_heads,), float("-inf"), device=DEV)
    out, st = run_gpu(qd, kd, vd, neg, bm, bn)
    assert out.dtype == torch.float16
    rep = parity.compare(qd, kd, vd, neg, bm, bn, True, out, st.skip_mask, st.block_max, lse_gpu=st.lse)
    assert rep.skipped == 0
    tau = binding.bsfa_calibrate(qd, kd, [0.5], block_m=bm, block_n=bn)[0]
    out, st = run_gpu(qd, kd, vd, tau.to(DEV), bm, bn)
    rep = parity.compare(qd, kd, vd, tau, bm, bn, True, out, st.skip_mask, st.block_max, lse_gpu=st.lse)
    assert rep.skipped > 0
    n = shp.seqlen - 37
    qr, kr, vr = (t[:, :n].contiguous() for t in (qd, kd, vd))
    out, st = run_gpu(qr, kr, vr, tau.to(DEV), bm, bn, dump=False)
    parity.compare(qr, kr, vr, tau, bm, bn, True, out, st.skip_mask)
    with pytest.raises(TypeError):
        binding.bsfa_forward(qd, kd.to(torch.bfloat16), vd, neg, block_m=bm, block_n=bn)


def test_forward_in_a_hip_graph(oracle):
    """bsfa_forward only enqueues kernels (the counters are cleared by a fill kernel, not a
    memset), so it can be captured: a captured launch is replayed three times on changing inputs,
    with eager work and synchronisation in between, and every replay must equal the eager result
    bit for bit."""
    shp = synth.Shape(1, 1024, 4, 2, 128, 128, 64)
    sets = [to_dev(*synth.tiny(100 + s, shp, n_boost=5)) for s in range(3)]
    q, k, v = (t.clone() for t in sets[0])
    tau = binding.bsfa_calibrate(q, k, [0.5])[0].to(DEV)
    out = torch.empty_like(q)
    st = binding.alloc_stats(q, 128, 64, counts=True, skip_mask=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside the capture
        binding.bsfa_forward(q, k, v, tau, out=out, skip_stats=st)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        binding.bsfa_forward(q, k, v, tau, out=out, skip_stats=st)
    for n, (qs, ks, vs) in enumerate(sets[::-1] + sets):
        q.copy_(qs); k.copy_(ks); v.copy_(vs)
        out.fill_(float("nan")); st.counts.fill_(-1); st.skip_mask.fill_(-1)
        g.replay()
        torch.cuda.synchronize()
        got, got_counts, got_mask = out.clone(), st.counts.clone(), st.skip_mask.clone()
        st2 = binding.alloc_stats(q, 128, 64, counts=True, skip_mask=True)
        ref = binding.bsfa_forward(qs, ks, vs, tau, skip_stats=st2)
        torch.cuda.synchronize()
        assert torch.equal(got, ref), "replay %d differs from the eager launch" % n
        assert torch.equal(got_counts, st2.counts) and torch.equal(got_mask, st2.skip_mask)
    parity.compare(q, k, v, tau, 128, 64, True, out, st.skip_mask)


def test_single_head_groups_gives_identical_results(oracle):
    """The tuning knob that stops pairing the heads of a GQA group changes the schedule, not the
    arithmetic: outputs, masks and counts are bit-identical, and both match the oracle."""
    shp = synth.Shape(1, 1024, 8, 2, 128, 128, 64)
    q, k, v = to_dev(*synth.tiny(71, shp, n_boost=5))
    tau = binding.bsfa_calibrate(q, k, [0.6])[0].to(DEV)
    res = []
    for single in (False, True):
        st = binding.alloc_stats(q, 128, 64, counts=True, skip_mask=True, block_max=True, lse=True)
        out = binding.bsfa_forward(q, k, v, tau, skip_stats=st, single_head_groups=single)
        torch.cuda.synchronize()
        res.append((out, st))
    (o0, s0), (o1, s1) = res
    assert torch.equal(o0, o1) and torch.equal(s0.skip_mask, s1.skip_mask) and torch.equal(s0.counts, s1.counts)
    assert torch.equal(s0.lse, s1.lse) and torch.equal(torch.nan_to_num(s0.block_max), torch.nan_to_num(s1.block_max))
    parity.compare(q, k, v, tau, 128, 64, True, o1, s1.skip_mask, s1.block_max, lse_gpu=s1.lse)


@pytest.mark.parametrize("case,dtype", [((1, 1152, 16, 8, 128, 128, 64), torch.bfloat16), ((2, 640, 4, 2, 64, 128, 64), torch.float16),
                                        ((1, 900, 6, 2, 128, 128, 64), torch.bfloat16)])
def test_workspace_path_is_bit_identical_to_in_place_v(case, dtype):
    """With a workspace V is first rewritten as transposed tiles and the second product reads it with
    full-width LDS reads; without one V is gathered in place with transposing reads.  Both feed the
    same numbers to the same MFMAs: outputs, masks and log-sum-exps must be equal bit for bit
    (paired heads, single heads, ragged length, a workspace that is too small)."""
    shp = synth.Shape(*case)
    q, k, v = (t.to(dtype).to(DEV) for t in synth.tiny(77, shp, n_boost=max(1, shp.m_kv // 3)))
    if case[1] == 900:
        q, k, v = (t[:, :870].contiguous() for t in (q, k, v))
    tau = binding.bsfa_calibrate(q, k, [0.5])[0].to(DEV)
    need = binding.forward_workspace_bytes(q, k)
    assert need >= v.numel() * 2
    ws = torch.full((need + 512,), 0xFF, dtype=torch.uint8, device=DEV)       # NaN bit patterns everywhere
    res = {}
    for name, kw in (("in_place", dict(workspace=None)), ("workspace", dict(workspace=ws[256:])),
                     ("workspace_single", dict(workspace=ws, single_head_groups=True)),
                     ("in_place_single", dict(workspace=None, single_head_groups=True))):
        st = binding.alloc_stats(q, 128, 64, counts=True, skip_mask=True, lse=True)
        out = binding.bsfa_forward(q, k, v, tau, skip_stats=st, **kw)
        torch.cuda.synchronize()
        res[name] = (out.clone(), st.skip_mask.clone(), st.lse.clone(), st.counts.clone())
    assert res["in_place"][3][..., 0].sum() > 0
    for name in ("workspace", "workspace_single", "in_place_single"):
        for a, b in zip(res["in_place"], res[name]):
            assert torch.equal(a, b), name
    with pytest.raises(binding.BsfaError) as e:
        binding.bsfa_forward(q, k, v, tau, workspace=ws[:need - 1024])
    assert e.value.status == -5


@pytest.mark.parametrize("qk_fp8", [False, True])
def test_running_max_predicate_matches_algorithm(oracle, qk_fp8):
    """(With qk_fp8 the oracle sees Q and K rounded to e4m3, the values the score product multiplies.)
    gate_mode = 1, the comparison predicate of Section 3, against its step-by-step oracle form:
    statistic per (tile, block) to 1e-4, decisions exactly (lambda is placed where no statistic of
    the oracle's own trajectory lies within 1e-3 of it, so no decision can legitimately flip and
    drag the running maximum with it), outputs within the usual tolerance of the exact softmax
    over the kept blocks."""
    shp = synth.Shape(1, 1024, 4, 2, 128, 128, 64)
    g = torch.Generator().manual_seed(5)
    u = torch.nn.functional.normalize(torch.randn(128, generator=g), dim=0)
    q = 3.0 * u + 0.5 * torch.randn(1, 1024, 4, 128, generator=g)
    k = torch.randn(1, 1024, 2, 128, generator=g)
    # block 0 sets a high running maximum; blocks 3 and 9 come within |lambda| of it, 6 and 12 do not
    for blk, amp in ((0, 40.0), (3, 36.0), (9, 36.0), (6, 30.0), (12, 30.0)):
        k[:, blk * 64:(blk + 1) * 64] += amp * u
    v = torch.randn(1, 1024, 2, 128, generator=g)
    qd, kd, vd = to_dev(q, k, v)
    qf, kf, vf = (t.float().cpu().numpy() for t in (qd, kd, vd))
    if qk_fp8:
        qf, kf = (_to_e4m3(t).float().cpu().numpy() for t in (qd, kd))
    lam0 = -2.0
    # oracle trajectories; move lambda away from any statistic that is too close
    def run_oracle(lam):
        res = {}
        for h in range(4):
            for i in range(shp.m_q):
                res[(h, i)] = oracle.alg1_tile_running_max(qf, kf, vf, lam, 0, h, i, 128, 64)
        return res
    lam = lam0
    for _ in range(20):
        res = run_oracle(lam)
        near = [abs(float(s) - lam) for r in res.values() for s in r[3].values()]
        if min(near) > (2e-2 if qk_fp8 else 2e-3):
            break
        lam -= 0.0137
    else:
        pytest.fail("no clear lambda found")
    lam_d = torch.full((4,), lam, device=DEV)
    st = binding.alloc_stats(qd, 128, 64, counts=True, skip_mask=True, block_max=True, lse=True)
    out = binding.bsfa_forward(qd, kd, vd, lam_d, skip_stats=st, gate_mode=1, qk_fp8=qk_fp8)
    torch.cuda.synchronize()
    mask = parity.unpack_mask(st.skip_mask.cpu().numpy(), shp.m_kv)[0]        # [h, i, j] True = skipped
    bmx = st.block_max.cpu().numpy()[0]
    o = out.float().cpu().numpy()[0]
    lse = st.lse.cpu().numpy()[0]
    n_skipped = 0
    for (h, i), (O, L, kept, stats) in res.items():
        n_reach = 2 * i + 2
        skipped = [j for j in range(n_reach) if j not in kept]
        assert list(np.nonzero(mask[h, i])[0]) == skipped, (h, i)
        n_skipped += len(skipped)
        # the statistic is a difference of two scores of magnitude ~40: 1e-4 absolute holds for the 16-bit
        # product; the fp8 MFMA sums its 64-term products in another order, 1e-4 relative to the scores
        tol = 4e-3 if qk_fp8 else 1e-4
        for j, s_ in stats.items():
            assert abs(bmx[h, i, j] - float(s_)) < tol
        assert np.isnan(bmx[h, i, len(stats):]).all()
        err = np.abs(o[i * 128:(i + 1) * 128, h] - O)
        assert err.max() <= parity.MAX_ABS and err.mean() <= parity.MEAN_ABS
        assert np.abs(lse[i * 128:(i + 1) * 128, h] - L).max() < 5e-3
    assert n_skipped > 20
    assert int(st.counts[0, :, 0].sum()) == n_skipped
    # the same call with gate_mode 0 takes the thresholds as T: a different mask
    st0 = binding.alloc_stats(qd, 128, 64, counts=True)
    binding.bsfa_forward(qd, kd, vd, lam_d, skip_stats=st0, qk_fp8=qk_fp8)
    torch.cuda.synchronize()
    assert int(st0.counts[0, :, 0].sum()) == 0            # every block maximum is far above -2
    kept_gate = sum(len([j for j in r[2] if j in r[3] and j > 0]) for r in res.values())
    assert kept_gate > 5                                  # and some gateable blocks behind the first survive
    with pytest.raises(binding.BsfaError):
        binding.bsfa_forward(qd, kd, vd, lam_d, gate_mode=2)


def _to_e4m3(t):
    """Round to fp8 e4m3 (nearest even) and widen back: every value is then exact in bf16."""
    return t.to(torch.float8_e4m3fn).to(torch.bfloat16)


@pytest.mark.parametrize("hq,hkv,n", [(4, 2, 1024), (6, 2, 870)])
def test_fp8_score_product(oracle, hq, hkv, n):
    """qk_fp8: the score product runs on fp8 (e4m3) copies of Q and K.  The kernel's rounding is round to
    nearest even, so on bf16 inputs it must agree with the oracle fed Q and K rounded the same way by
    torch (block maxima to 1e-4, masks outside the band, outputs within the usual tolerances), and on
    inputs that already are fp8 values it changes nothing about what is compared.  Paired and single
    heads, ragged length, dense and gated, thresholds from bsfa_calibrate in the same mode."""
    shp = synth.Shape(1, 1024, hq, hkv, 128, 128, 64)
    q, k, v = (t.to(torch.bfloat16).to(DEV) for t in synth.tiny(91, shp, n_boost=5))
    q, k, v = (t[:, :n].contiguous() for t in (q, k, v))
    q8, k8 = _to_e4m3(q), _to_e4m3(k)
    assert not torch.equal(q8, q)
    tau = binding.bsfa_calibrate(q, k, [0.5], qk_fp8=True)[0]
    # calibration in fp8 mode = order statistic of the fp8-rounded problem's block maxima (the 16-bit
    # product of the same values sums in another order: equal to rounding)
    tau_ref = binding.bsfa_calibrate(q8, k8, [0.5])[0]
    assert torch.allclose(tau, tau_ref, rtol=0, atol=3e-4)
    neg = torch.full((hq,), float("-inf"))
    for thr in (neg, tau):
        for inputs in ((q, k), (q8, k8)):
            st = binding.alloc_stats(q, 128, 64, counts=True, skip_mask=True, block_max=True, lse=True)
            out = binding.bsfa_forward(inputs[0], inputs[1], v, thr.to(DEV), skip_stats=st, qk_fp8=True)
            torch.cuda.synchronize()
            rep = parity.compare(q8, k8, v, thr, 128, 64, True, out, st.skip_mask, st.block_max, lse_gpu=st.lse)
            assert rep.mask_mismatch <= rep.in_band
        if thr is tau:
            assert rep.skipped > 0
    # and the 16-bit path on the rounded inputs gives the same masks (same scores up to summation order)
    st2 = binding.alloc_stats(q, 128, 64, counts=True, skip_mask=True)
    binding.bsfa_forward(q8, k8, v, tau.to(DEV), skip_stats=st2)
    torch.cuda.synchronize()
    assert (st2.counts[..., 0] - st.counts[..., 0]).abs().sum() <= rep.in_band
    with pytest.raises(binding.BsfaError) as e:
        binding.bsfa_forward(q, k, v, tau.to(DEV), qk_fp8=True, workspace=None)
    assert e.value.status == -5
