"""Host-side checks of the seeded input recipes (no method arithmetic involved)."""
import torch

from paper_2512_07011_amd import synth


def test_tiny_is_seeded_and_boosts_whole_blocks():
    a = synth.tiny(3)
    b = synth.tiny(3)
    c = synth.tiny(4)
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    assert not torch.equal(a[1], c[1])
    q, k, v = a
    assert q.shape == (1, 512, 2, 64) and k.shape == (1, 512, 2, 64) and q.dtype == torch.float32
    _, k0, _ = synth.tiny(3, n_boost=0)
    diff = (k - k0).abs().amax(dim=-1)[0]                        # [N, Hkv]
    for h in range(2):
        blocks = diff[:, h].view(8, 64)
        changed = (blocks > 0).all(dim=1)
        assert changed.sum() == 4 and ((blocks > 0).any(dim=1) == changed).all()


def test_llama_layer_shapes_sink_and_needles():
    shp = synth.llama_shape(2048)
    q, k, v = synth.llama_layer(5, shp)
    assert q.shape == (1, 2048, 32, 128) and k.shape == (1, 2048, 8, 128) and v.shape == k.shape
    assert q.dtype == k.dtype == v.dtype == torch.bfloat16
    q2, k2, _ = synth.llama_layer(5, shp)
    assert torch.equal(k, k2) and torch.equal(q, q2)
    _, kp, _ = synth.llama_layer(5, shp, sink_gain=0.0, n_needles=0, dtype=torch.float32)
    _, ks, _ = synth.llama_layer(5, shp, n_needles=0, dtype=torch.float32)
    d = (ks - kp).norm(dim=-1)[0]                                # [N, Hkv]
    assert torch.allclose(d[:64], torch.full_like(d[:64], 4.0), atol=1e-4) and (d[64:] == 0).all()
    _, kn, _ = synth.llama_layer(5, shp, sink_gain=0.0, dtype=torch.float32)
    touched = ((kn - kp).abs().amax(dim=-1)[0] > 0)              # [N, Hkv]
    # needles of tile i live in gateable blocks only: none at or after the last tile's first row
    assert not touched[(shp.m_q - 1) * shp.block_m:].any()
    n_expected = sum(min(8, synth.n_gateable(i, 128, 64)) for i in range(1, shp.m_q)) * 32
    assert 0.8 * n_expected <= touched.sum() <= n_expected      # collisions only lower the count


def test_n_gateable():
    assert [synth.n_gateable(i, 128, 64) for i in range(4)] == [0, 2, 4, 6]
    assert [synth.n_gateable(i, 64, 64) for i in range(4)] == [0, 1, 2, 3]
    assert [synth.n_gateable(i, 32, 64) for i in range(5)] == [0, 0, 1, 1, 2]
