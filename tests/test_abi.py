"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the
header declares, and rejects bad arguments with the documented codes before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2512_07011_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "bsfa.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2512_07011_amd import build
        build.build_lib()
    return binding.lib()


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(bsfa_[a-z_]+)\s*\(", src)))


def test_header_functions_are_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS), names
    for n in names:
        assert getattr(lib, n) is not None


def good_problem(**kw):
    p = binding.bsfa_problem()
    p.batch, p.n_q_heads, p.n_kv_heads, p.seqlen, p.head_dim, p.block_m, p.block_n = 1, 4, 2, 512, 128, 128, 64
    for t, h in (("q", 4), ("k", 2), ("v", 2), ("o", 4)):
        setattr(p, t + "_stride_b", 512 * h * 128)
        setattr(p, t + "_stride_n", h * 128)
        setattr(p, t + "_stride_h", 128)
    for k, v in kw.items():
        setattr(p, k, v)
    return p


FAKE = ctypes.c_void_p(0x1000)      # never dereferenced: validation fails first


@pytest.mark.parametrize("kw, code", [
    (dict(batch=0), -2), (dict(seqlen=0), -2), (dict(n_q_heads=3), -2), (dict(dtype=7), -3),
    (dict(head_dim=96), -4), (dict(block_m=96), -4), (dict(block_n=32), -4), (dict(block_m=256), -4),
    (dict(q_stride_n=516), -2), (dict(k_stride_h=64), -2), (dict(thresholds_per_tile=2), -2),
    (dict(o_stride_b=-8), -2), (dict(threshold_tiles=-1), -2), (dict(seqlens=0x1002), -2), (dict(single_head_groups=2), -2),
])
def test_forward_rejects_bad_problems(lib, kw, code):
    p = good_problem(**kw)
    rc = lib.bsfa_forward(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, 1, FAKE, None, None)
    assert rc == code, (kw, rc, lib.bsfa_last_error())
    assert lib.bsfa_last_error() != b""
    assert lib.bsfa_calibrate_workspace_bytes(ctypes.byref(p)) == 0


def test_ragged_lengths_need_the_causal_mask(lib):
    """Without the causal mask padded keys would be visible: a sequence that does not fill its
    last block, or per-element lengths, are rejected there (and accepted with the mask: checked on
    the GPU, where the pointers are real)."""
    for kw in (dict(seqlen=500), dict(seqlen=544), dict(seqlens=0x1000)):
        p = good_problem(**kw)
        assert lib.bsfa_forward(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, 0, FAKE, None, None) == -2, kw
    # the workspace query assumes the causal mask: ceil(500/128) x ceil(500/64) maxima per head
    assert lib.bsfa_calibrate_workspace_bytes(ctypes.byref(good_problem(seqlen=500))) >= 4 * 4 * 8 * 4


def test_null_and_alignment(lib):
    p = good_problem()
    assert lib.bsfa_forward(None, FAKE, FAKE, FAKE, FAKE, 1, FAKE, None, None) == -1
    assert lib.bsfa_forward(ctypes.byref(p), None, FAKE, FAKE, FAKE, 1, FAKE, None, None) == -1
    assert lib.bsfa_forward(ctypes.byref(p), FAKE, FAKE, FAKE, None, 1, FAKE, None, None) == -1
    assert lib.bsfa_forward(ctypes.byref(p), ctypes.c_void_p(0x1008), FAKE, FAKE, FAKE, 1, FAKE, None, None) == -2


def test_calibrate_argument_checks(lib):
    p = good_problem()
    need = lib.bsfa_calibrate_workspace_bytes(ctypes.byref(p))
    assert need >= 4 * 4 * 8 * 4
    fr = (ctypes.c_float * 2)(0.5, 0.25)
    out = (ctypes.c_float * 8)()
    assert lib.bsfa_calibrate(ctypes.byref(p), FAKE, FAKE, 1, fr, 2, out, None, 0, None) == -5
    assert lib.bsfa_calibrate(ctypes.byref(p), FAKE, FAKE, 1, fr, 2, out, FAKE, need - 1, None) == -5
    bad = (ctypes.c_float * 1)(1.5)
    assert lib.bsfa_calibrate(ctypes.byref(p), FAKE, FAKE, 1, bad, 1, out, FAKE, need, None) == -2
    assert lib.bsfa_calibrate(ctypes.byref(p), FAKE, FAKE, 1, fr, 0, out, FAKE, need, None) == -2
    assert lib.bsfa_calibrate(ctypes.byref(p), FAKE, FAKE, 1, None, 1, out, FAKE, need, None) == -1
    pt = good_problem(thresholds_per_tile=1)
    assert lib.bsfa_calibrate(ctypes.byref(pt), FAKE, FAKE, 1, fr, 2, out, FAKE, need, None) == -4


def test_calibrate_topk_argument_checks(lib):
    p = good_problem()
    need = lib.bsfa_calibrate_workspace_bytes(ctypes.byref(p))
    ks = (ctypes.c_int32 * 2)(4, 8)
    out = (ctypes.c_float * (2 * 4 * 4))()
    assert lib.bsfa_calibrate_topk(ctypes.byref(p), FAKE, FAKE, 1, ks, 2, 0, out, None, 0, None) == -5
    assert lib.bsfa_calibrate_topk(ctypes.byref(p), FAKE, FAKE, 1, None, 2, 0, out, FAKE, need, None) == -1
    assert lib.bsfa_calibrate_topk(ctypes.byref(p), FAKE, FAKE, 1, ks, 0, 0, out, FAKE, need, None) == -2
    assert lib.bsfa_calibrate_topk(ctypes.byref(p), FAKE, FAKE, 1, ks, 2, -1, out, FAKE, need, None) == -2
    neg = (ctypes.c_int32 * 1)(-3)
    assert lib.bsfa_calibrate_topk(ctypes.byref(p), FAKE, FAKE, 1, neg, 1, 0, out, FAKE, need, None) == -2
    assert lib.bsfa_calibrate_topk(ctypes.byref(good_problem(seqlen=500)), FAKE, FAKE, 0, ks, 2, 0, out, FAKE, need, None) == -2
    assert lib.bsfa_calibrate_topk(ctypes.byref(good_problem(seqlens=0x1000)), FAKE, FAKE, 1, ks, 2, 0, out, FAKE, need, None) == -4


def test_query_build_and_status_strings(lib):
    tiles = binding.bsfa_query_build()
    assert (128, 64, 128) in tiles and (64, 64, 64) in tiles
    assert all(bn == 64 for _, bn, _ in tiles)
    for code, name in binding.STATUS_NAMES.items():
        assert lib.bsfa_status_string(code) == name.encode()
    assert lib.bsfa_status_string(-99) == b"BSFA_ERR_UNKNOWN"


def test_binding_refuses_cpu_tensors():
    import torch
    q = torch.zeros(1, 128, 2, 128, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        binding.bsfa_forward(q, q, q, torch.zeros(2))
