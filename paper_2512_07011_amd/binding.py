"""ctypes binding of libbsfa.so (see include/bsfa.h).  Argument marshalling only: every step of
the attention path runs inside the library's HIP kernels.  PyTorch supplies device memory and
the current stream; there is no fallback — if the library is missing or a call fails, this
module raises."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbsfa.so")

BSFA_OK = 0
STATUS_NAMES = {0: "BSFA_OK", -1: "BSFA_ERR_NULL", -2: "BSFA_ERR_SHAPE", -3: "BSFA_ERR_DTYPE",
                -4: "BSFA_ERR_UNSUPPORTED", -5: "BSFA_ERR_WORKSPACE", -6: "BSFA_ERR_HIP"}
EXPORTS = ["bsfa_forward", "bsfa_forward_workspace_bytes", "bsfa_calibrate", "bsfa_calibrate_noalloc",
           "bsfa_calibrate_noalloc_max_values", "bsfa_calibrate_topk",
           "bsfa_calibrate_workspace_bytes", "bsfa_query_build",
           "bsfa_mfma_rate_probe", "bsfa_mfma_rate_probe_sink_bytes", "bsfa_mfma_rate_probe_flops",
           "bsfa_status_string", "bsfa_last_error"]


DTYPES = {torch.bfloat16: 0, torch.float16: 1}       # bsfa_dtype


def _same_16bit(name, *ts):
    if ts[0].dtype not in DTYPES or any(t.dtype != ts[0].dtype for t in ts):
        raise TypeError("%s: tensors must all be bfloat16 or all float16" % name)


class BsfaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("%s: %s" % (STATUS_NAMES.get(status, str(status)), message))
        self.status = status


class bsfa_problem(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("batch", "n_q_heads", "n_kv_heads", "seqlen", "head_dim", "block_m", "block_n")] + \
               [(n, ctypes.c_int64) for n in
                ("q_stride_b", "q_stride_n", "q_stride_h", "k_stride_b", "k_stride_n", "k_stride_h",
                 "v_stride_b", "v_stride_n", "v_stride_h", "o_stride_b", "o_stride_n", "o_stride_h")] + \
               [("dtype", ctypes.c_int32), ("thresholds_per_tile", ctypes.c_int32),
                ("threshold_tiles", ctypes.c_int32), ("seqlens", ctypes.c_void_p),
                ("single_head_groups", ctypes.c_int32), ("gate_mode", ctypes.c_int32), ("qk_fp8", ctypes.c_int32), ("workspace", ctypes.c_void_p),
                ("workspace_bytes", ctypes.c_int64)]


class bsfa_skip_stats(ctypes.Structure):
    _fields_ = [("counts", ctypes.c_void_p), ("skip_mask", ctypes.c_void_p), ("block_max", ctypes.c_void_p),
                ("lse", ctypes.c_void_p)]


_lib = None


def lib() -> ctypes.CDLL:
    """Opens libbsfa.so (built in-tree by build.build_lib / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s is missing: build it with `python -m paper_2512_07011_amd.build` "
                "(there is no fallback path)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        L.bsfa_forward.restype = ctypes.c_int
        L.bsfa_forward.argtypes = [ctypes.POINTER(bsfa_problem), vp, vp, vp, vp, ctypes.c_int, vp,
                                   ctypes.POINTER(bsfa_skip_stats), vp]
        L.bsfa_calibrate.restype = ctypes.c_int
        L.bsfa_calibrate.argtypes = [ctypes.POINTER(bsfa_problem), vp, vp, ctypes.c_int,
                                     ctypes.POINTER(ctypes.c_float), ctypes.c_int,
                                     ctypes.POINTER(ctypes.c_float), vp, ctypes.c_size_t, vp]
        L.bsfa_calibrate_noalloc.restype = ctypes.c_int
        L.bsfa_calibrate_noalloc.argtypes = [ctypes.POINTER(bsfa_problem), vp, vp, ctypes.c_int,
                                             ctypes.POINTER(ctypes.c_float), ctypes.c_int, vp, vp]
        L.bsfa_calibrate_noalloc_max_values.restype = ctypes.c_size_t
        L.bsfa_calibrate_noalloc_max_values.argtypes = []
        L.bsfa_calibrate_topk.restype = ctypes.c_int
        L.bsfa_calibrate_topk.argtypes = [ctypes.POINTER(bsfa_problem), vp, vp, ctypes.c_int,
                                          ctypes.POINTER(ctypes.c_int32), ctypes.c_int, ctypes.c_int,
                                          ctypes.POINTER(ctypes.c_float), vp, ctypes.c_size_t, vp]
        L.bsfa_calibrate_workspace_bytes.restype = ctypes.c_size_t
        L.bsfa_calibrate_workspace_bytes.argtypes = [ctypes.POINTER(bsfa_problem)]
        L.bsfa_forward_workspace_bytes.restype = ctypes.c_size_t
        L.bsfa_forward_workspace_bytes.argtypes = [ctypes.POINTER(bsfa_problem)]
        i32p = ctypes.POINTER(ctypes.c_int32)
        L.bsfa_query_build.restype = ctypes.c_int
        L.bsfa_query_build.argtypes = [i32p, i32p, i32p, ctypes.c_int]
        L.bsfa_mfma_rate_probe.restype = ctypes.c_int
        L.bsfa_mfma_rate_probe.argtypes = [vp, vp, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, vp]
        L.bsfa_mfma_rate_probe_sink_bytes.restype = ctypes.c_size_t
        L.bsfa_mfma_rate_probe_sink_bytes.argtypes = [ctypes.c_int]
        L.bsfa_mfma_rate_probe_flops.restype = ctypes.c_double
        L.bsfa_mfma_rate_probe_flops.argtypes = [ctypes.c_int, ctypes.c_int]
        L.bsfa_status_string.restype = ctypes.c_char_p
        L.bsfa_status_string.argtypes = [ctypes.c_int]
        L.bsfa_last_error.restype = ctypes.c_char_p
        L.bsfa_last_error.argtypes = []
        _lib = L
    return _lib


def _check(status: int):
    if status != BSFA_OK:
        raise BsfaError(status, lib().bsfa_last_error().decode())


def make_problem(q: torch.Tensor, k: torch.Tensor, v: Optional[torch.Tensor], out: Optional[torch.Tensor],
                 block_m: int, block_n: int, thresholds_per_tile: bool = False, threshold_tiles: int = 0,
                 seqlens: Optional[torch.Tensor] = None, single_head_groups: bool = False) -> bsfa_problem:
    """Descriptor for [B, N, H, d] views (any strides with a contiguous last dimension)."""
    B, N, Hq, d = q.shape
    p = bsfa_problem()
    p.batch, p.seqlen, p.n_q_heads, p.n_kv_heads, p.head_dim = B, N, Hq, k.shape[2], d
    p.block_m, p.block_n = block_m, block_n
    for name, t in (("q", q), ("k", k), ("v", v if v is not None else k), ("o", out if out is not None else q)):
        if t.stride(3) != 1:
            raise ValueError("%s: head dimension must be contiguous" % name)
        setattr(p, name + "_stride_b", t.stride(0))
        setattr(p, name + "_stride_n", t.stride(1))
        setattr(p, name + "_stride_h", t.stride(2))
    p.dtype = DTYPES[q.dtype]
    p.thresholds_per_tile = int(thresholds_per_tile)
    p.threshold_tiles = int(threshold_tiles)
    p.single_head_groups = int(bool(single_head_groups))
    if seqlens is not None:
        if seqlens.dtype != torch.int32 or not seqlens.is_contiguous() or tuple(seqlens.shape) != (B,) or not seqlens.is_cuda:
            raise TypeError("bsfa: seqlens must be a contiguous int32 GPU tensor of shape [batch]")
        p.seqlens = seqlens.data_ptr()
    return p


def n_tiles(n: int, block: int) -> int:
    """Query tiles / key blocks of a sequence of n tokens (the last one may be partial)."""
    return -(-n // block)


@dataclass
class SkipStats:
    counts: Optional[torch.Tensor] = None      # [B, Hq, 3] int64: skipped, gateable, reachable
    skip_mask: Optional[torch.Tensor] = None   # [B, Hq, M_Q, ceil(M_KV/32)] int32 bit mask
    block_max: Optional[torch.Tensor] = None   # [B, Hq, M_Q, M_KV] fp32, NaN where not gateable
    lse: Optional[torch.Tensor] = None         # [B, N, Hq] fp32, log-sum-exp over the kept blocks


def alloc_stats(q: torch.Tensor, block_m: int, block_n: int, counts=True, skip_mask=False, block_max=False,
                lse=False) -> SkipStats:
    B, N, Hq, _ = q.shape
    mq, mkv = n_tiles(N, block_m), n_tiles(N, block_n)
    s = SkipStats()
    if counts:
        s.counts = torch.empty(B, Hq, 3, dtype=torch.int64, device=q.device)
    if skip_mask:
        s.skip_mask = torch.empty(B, Hq, mq, (mkv + 31) // 32, dtype=torch.int32, device=q.device)
    if block_max:
        s.block_max = torch.empty(B, Hq, mq, mkv, dtype=torch.float32, device=q.device)
    if lse:
        s.lse = torch.empty(B, N, Hq, dtype=torch.float32, device=q.device)
    return s


_workspaces = {}


def _cached_workspace(device, nbytes: int):
    """One growing scratch tensor per device for callers that do not manage the forward workspace
    themselves (calls that overlap on different streams must pass their own)."""
    if nbytes == 0:
        return None
    w = _workspaces.get(device)
    if w is None or w.numel() < nbytes:
        w = torch.empty(nbytes, dtype=torch.uint8, device=device)
        _workspaces[device] = w
    return w


def forward_workspace_bytes(q: torch.Tensor, k: torch.Tensor, block_m: int = 128, block_n: int = 64,
                            qk_fp8: bool = False) -> int:
    """Bytes of workspace bsfa_forward can use for these shapes (0: none)."""
    p = make_problem(q, k, None, None, block_m, block_n)
    p.qk_fp8 = int(bool(qk_fp8))
    return int(lib().bsfa_forward_workspace_bytes(ctypes.byref(p)))


def _dev_check(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("bsfa: tensors must live on the GPU")


def bsfa_forward(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, thresholds: torch.Tensor,
                 causal: bool = True, out: Optional[torch.Tensor] = None,
                 skip_stats: Optional[SkipStats] = None, block_m: int = 128, block_n: int = 64,
                 stream: Optional[torch.cuda.Stream] = None,
                 seqlens: Optional[torch.Tensor] = None, single_head_groups: bool = False,
                 workspace=True, gate_mode: int = 0, qk_fp8: bool = False) -> torch.Tensor:
    """out = block-sparse attention of bf16 (or fp16) q [B,N,Hq,d], k, v [B,N,Hkv,d]; thresholds fp32 on the
    GPU, [Hq] or [Hq, T] (T tiles calibrated; later tiles use the last one).  ``seqlens`` (int32
    GPU tensor [B], causal only) gives each batch element its own length.  ``workspace``: a uint8
    GPU tensor of at least forward_workspace_bytes(...) bytes, True (a cached tensor per device is
    used) or False/None (no workspace: V is read in place).  ``gate_mode`` 1 selects the
    running-maximum comparison predicate (thresholds then hold its lambda).  Enqueues on ``stream`` (default:
    torch's current stream)."""
    _dev_check(q, k, v, thresholds, out)
    _same_16bit("bsfa_forward", q, k, v, *([out] if out is not None else []))
    if thresholds.dtype != torch.float32 or not thresholds.is_contiguous():
        raise TypeError("bsfa_forward: thresholds must be contiguous float32")
    per_tile = thresholds.dim() == 2
    B, N, Hq, d = q.shape
    if thresholds.dim() not in (1, 2) or thresholds.shape[0] != Hq or (per_tile and thresholds.shape[1] < 1):
        raise ValueError("bsfa_forward: thresholds shape %s, expected [Hq] or [Hq, tiles]" % (tuple(thresholds.shape),))
    if out is None:
        out = torch.empty_like(q)
    p = make_problem(q, k, v, out, block_m, block_n, per_tile, thresholds.shape[1] if per_tile else 0, seqlens,
                     single_head_groups)
    p.gate_mode = int(gate_mode)
    p.qk_fp8 = int(bool(qk_fp8))
    if workspace is True:
        workspace = _cached_workspace(q.device, lib().bsfa_forward_workspace_bytes(ctypes.byref(p)))
    if workspace is not None and workspace is not False:
        _dev_check(workspace)
        p.workspace = workspace.data_ptr()
        p.workspace_bytes = workspace.numel() * workspace.element_size()
    st = None
    if skip_stats is not None:
        st = bsfa_skip_stats(
            skip_stats.counts.data_ptr() if skip_stats.counts is not None else None,
            skip_stats.skip_mask.data_ptr() if skip_stats.skip_mask is not None else None,
            skip_stats.block_max.data_ptr() if skip_stats.block_max is not None else None,
            skip_stats.lse.data_ptr() if skip_stats.lse is not None else None)
    s = stream if stream is not None else torch.cuda.current_stream(q.device)
    _check(lib().bsfa_forward(ctypes.byref(p), q.data_ptr(), k.data_ptr(), v.data_ptr(), thresholds.data_ptr(),
                              int(bool(causal)), out.data_ptr(), ctypes.byref(st) if st is not None else None,
                              ctypes.c_void_p(s.cuda_stream)))
    return out


def bsfa_calibrate(q: torch.Tensor, k: torch.Tensor, target_skip_fractions: Sequence[float],
                   causal: bool = True, block_m: int = 128, block_n: int = 64,
                   workspace: Optional[torch.Tensor] = None,
                   stream: Optional[torch.cuda.Stream] = None,
                   seqlens: Optional[torch.Tensor] = None, qk_fp8: bool = False) -> torch.Tensor:
    """Per-head thresholds for each target skip fraction: CPU float32 tensor [n_levels, Hq]."""
    _dev_check(q, k, workspace)
    _same_16bit("bsfa_calibrate", q, k)
    p = make_problem(q, k, None, None, block_m, block_n, seqlens=seqlens)
    p.qk_fp8 = int(bool(qk_fp8))
    need = lib().bsfa_calibrate_workspace_bytes(ctypes.byref(p))
    if need == 0:
        _check(lib().bsfa_calibrate(ctypes.byref(p), q.data_ptr(), k.data_ptr(), int(bool(causal)), None, 0, None, None, 0, None))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    n = len(target_skip_fractions)
    fr = (ctypes.c_float * n)(*[float(f) for f in target_skip_fractions])
    outp = (ctypes.c_float * (n * q.shape[2]))()
    s = stream if stream is not None else torch.cuda.current_stream(q.device)
    _check(lib().bsfa_calibrate(ctypes.byref(p), q.data_ptr(), k.data_ptr(), int(bool(causal)), fr, n, outp,
                                workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                ctypes.c_void_p(s.cuda_stream)))
    return torch.tensor(list(outp), dtype=torch.float32).view(n, q.shape[2])


def bsfa_calibrate_noalloc(q: torch.Tensor, k: torch.Tensor, target_skip_fractions: Sequence[float],
                           thresholds_out: torch.Tensor, causal: bool = True, block_m: int = 128, block_n: int = 64,
                           stream: Optional[torch.cuda.Stream] = None,
                           seqlens: Optional[torch.Tensor] = None) -> torch.Tensor:
    """bsfa_calibrate without allocations: the thresholds go to ``thresholds_out``, a contiguous
    float32 GPU tensor [n_levels, Hq] the caller provides; kernels are only enqueued."""
    _dev_check(q, k, thresholds_out)
    _same_16bit("bsfa_calibrate_noalloc", q, k)
    n = len(target_skip_fractions)
    if thresholds_out.dtype != torch.float32 or not thresholds_out.is_contiguous() or tuple(thresholds_out.shape) != (n, q.shape[2]):
        raise TypeError("bsfa_calibrate_noalloc: thresholds_out must be contiguous float32 [n_levels, Hq]")
    p = make_problem(q, k, None, None, block_m, block_n, seqlens=seqlens)
    fr = (ctypes.c_float * n)(*[float(f) for f in target_skip_fractions])
    s = stream if stream is not None else torch.cuda.current_stream(q.device)
    _check(lib().bsfa_calibrate_noalloc(ctypes.byref(p), q.data_ptr(), k.data_ptr(), int(bool(causal)), fr, n,
                                        thresholds_out.data_ptr(), ctypes.c_void_p(s.cuda_stream)))
    return thresholds_out


def mfma_rate_probe(operands: torch.Tensor, workgroups: int, iters: int, sink: Optional[torch.Tensor] = None,
                    stream: Optional[torch.cuda.Stream] = None) -> float:
    """Enqueues the matrix-instruction rate probe (measurement utility) on ``operands`` (4096 float32 values on
    the GPU) and returns the floating-point operations it performs; the caller times it with events."""
    if not operands.is_cuda or operands.dtype != torch.float32 or not operands.is_contiguous() or operands.numel() < 4096:
        raise TypeError("mfma_rate_probe: operands must be a contiguous float32 GPU tensor of at least 4096 values")
    need = lib().bsfa_mfma_rate_probe_sink_bytes(int(workgroups))
    if sink is None:
        sink = torch.empty(max(need, 4) // 4, dtype=torch.float32, device=operands.device)
    s = stream if stream is not None else torch.cuda.current_stream(operands.device)
    _check(lib().bsfa_mfma_rate_probe(operands.data_ptr(), sink.data_ptr(), sink.numel() * sink.element_size(),
                                      int(workgroups), int(iters), ctypes.c_void_p(s.cuda_stream)))
    return float(lib().bsfa_mfma_rate_probe_flops(int(workgroups), int(iters)))


def bsfa_calibrate_topk(samples, ks: Sequence[int], causal: bool = True, block_m: int = 128, block_n: int = 64,
                        stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Per-query-tile thresholds for each sparsity level k (number of retained gateable blocks),
    averaged over the calibration samples: CPU float32 tensor [n_levels, Hq, ceil(N/block_m)].
    ``samples`` is a list of (q, k) pairs of equal shape; every batch element is one sample."""
    n = len(ks)
    out = None
    ws = None
    done = 0
    kk = (ctypes.c_int32 * n)(*[int(x) for x in ks])
    for q, k in samples:
        _dev_check(q, k)
        _same_16bit("bsfa_calibrate_topk", q, k)
        p = make_problem(q, k, None, None, block_m, block_n)
        need = lib().bsfa_calibrate_workspace_bytes(ctypes.byref(p))
        if ws is None or ws.numel() < need:
            ws = torch.empty(max(need, 1), dtype=torch.uint8, device=q.device)
        if out is None:
            out = (ctypes.c_float * (n * q.shape[2] * n_tiles(q.shape[1], block_m)))()
        s = stream if stream is not None else torch.cuda.current_stream(q.device)
        _check(lib().bsfa_calibrate_topk(ctypes.byref(p), q.data_ptr(), k.data_ptr(), int(bool(causal)), kk, n, done,
                                         out, ws.data_ptr(), ws.numel(), ctypes.c_void_p(s.cuda_stream)))
        done += q.shape[0]
    q0 = samples[0][0]
    return torch.tensor(list(out), dtype=torch.float32).view(n, q0.shape[2], n_tiles(q0.shape[1], block_m))


def bsfa_query_build():
    """List of (block_m, block_n, head_dim) triples the library was built for."""
    n = lib().bsfa_query_build(None, None, None, 0)
    bm, bn, hd = ((ctypes.c_int32 * n)() for _ in range(3))
    lib().bsfa_query_build(bm, bn, hd, n)
    return [(bm[i], bn[i], hd[i]) for i in range(n)]
