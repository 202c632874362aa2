"""The entry point that allocates nothing, bsfa_calibrate_noalloc, against bsfa_calibrate: same
thresholds bit for bit, on two calls in a row (the second on a smaller input, so that whatever the
first call left in the library's built-in scratch array must not leak into it), and its limits."""
import pytest
import torch

from paper_2512_07011_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
FR = [0.0, 0.1, 0.25, 0.5, 0.75, 0.9, 0.97, 1.0, 0.33, 0.66]        # more than one selection round


def _case(shape, seed, n=None):
    q, k, _ = synth.llama_layer(seed, shape, device=DEV) if shape.head_dim == 128 and shape.n_q_heads == 32 else \
        [t.to(torch.bfloat16).to(DEV) for t in synth.tiny(seed, shape, n_boost=max(1, shape.m_kv // 3))]
    if n is not None:
        q, k = q[:, :n].contiguous(), k[:, :n].contiguous()
    return q, k


def test_noalloc_matches_calibrate_twice_in_a_row():
    big = _case(synth.llama_shape(8192), 5)                          # 32 heads, 64 x 128 tiles per head
    small = _case(synth.Shape(2, 1024, 8, 2, 64, 128, 64), 6, n=900)   # batch 2, ragged, d = 64
    for q, k in (big, small):
        ref = binding.bsfa_calibrate(q, k, FR)                       # host tensor [levels, Hq]
        out = torch.full((len(FR), q.shape[2]), float("nan"), device=DEV)
        binding.bsfa_calibrate_noalloc(q, k, FR, out)
        torch.cuda.synchronize()
        got = out.cpu()
        assert torch.isneginf(got[0]).all() and torch.isposinf(got[7]).all()
        assert torch.equal(got, ref), (got - ref).abs().max()
        assert torch.isfinite(got[1:7]).all() and (got[1:7].diff(dim=0) >= 0).all()


def test_noalloc_limits_and_stream():
    q, k = _case(synth.Shape(1, 512, 4, 2, 64, 128, 64), 7)
    out = torch.empty(2, 4, device=DEV)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    binding.bsfa_calibrate_noalloc(q, k, [0.3, 0.6], out, stream=s)
    s.synchronize()
    assert torch.equal(out.cpu(), binding.bsfa_calibrate(q, k, [0.3, 0.6]))
    # 32 heads at 64K tokens: 16 Mi block maxima, four times what the built-in scratch array holds
    shp = synth.llama_shape(65536)
    qq = torch.empty(1, 65536, 32, 128, dtype=torch.bfloat16, device=DEV)
    kk = torch.empty(1, 65536, 8, 128, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(binding.BsfaError) as e:
        binding.bsfa_calibrate_noalloc(qq, kk, [0.5], torch.empty(1, 32, device=DEV))
    assert e.value.status == -5 and "scratch" in str(e.value)
    assert binding.lib().bsfa_calibrate_noalloc_max_values() == (16 << 20) // 4
