"""CPU oracle of the Block-Sparse FlashAttention forward pass.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this module;
the product path never does, and nothing here imports the HIP binding.

Two independent forms of the same result live here:

* ``forward`` / ``forward_items``: ctypes wrapper over ``bsfa_oracle.c`` — the definition
  (exact softmax attention restricted to the key blocks the gate keeps; Sections 2.1 and 4.1,
  Eq. 5-6), fp64 arithmetic on fp32 inputs.
* ``alg1_tile``: Algorithm 1 taken step by step in its own order and notation (running
  ``m``, ``l``, un-scaled accumulator, per-block gate), numpy fp64, small inputs only.  It
  visits the gateable blocks in any order the caller gives, which is what pins the claim that
  the two forms agree.

``alg1_tile_running_max`` is the same loop with the comparison predicate of Section 3 (local
row maxima against the running maxima) in place of the paper's gate.

``calibrate`` is the per-head threshold rule: an order statistic of the block maxima of the
gateable tiles (Section 4.2 sorts blocks by their maximum and picks the threshold retaining a
target count; the per-head quantile is the reduction of that rule over query positions).
``calibrate_topk`` is Section 4.2's rule itself: per query tile the k-th largest block
maximum, averaged over calibration samples.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bsfa_oracle.c")
_LIB = os.path.join(_HERE, "libbsfa_oracle.so")

CLS_UNREACHABLE, CLS_SKIPPED, CLS_KEPT, CLS_DIAGONAL = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP over independent query tiles)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        try:
            subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11",
                                   "-o", tmp, _SRC, "-lm"])
            os.replace(tmp, _LIB)
        finally:
            if os.path.exists(tmp):
                os.remove(tmp)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        fp = ctypes.POINTER(ctypes.c_float)
        lib.bsfa_oracle_items.restype = ctypes.c_int
        lib.bsfa_oracle_items.argtypes = [
            fp, fp, fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, fp, ctypes.c_int,
            ctypes.POINTER(ctypes.c_int32), ctypes.c_int, ctypes.POINTER(ctypes.c_uint8),
            fp, fp, ctypes.POINTER(ctypes.c_uint8), ctypes.POINTER(ctypes.c_double), fp]
        lib.bsfa_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the C oracle will use."""
    return int(_load().bsfa_oracle_threads())


def _f32(a) -> np.ndarray:
    """fp32 contiguous numpy view of a numpy array or a CPU torch tensor (bf16 widened)."""
    if hasattr(a, "detach"):
        a = a.detach().cpu().float().numpy()
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty)) if a is not None else None


@dataclass
class ItemResult:
    items: np.ndarray      # [n][3] (b, h, i)
    out: np.ndarray        # [n][BM][d] fp32
    bmax: np.ndarray       # [n][M_KV] fp32, NaN where not gateable
    cls: np.ndarray        # [n][M_KV] uint8: 0 unreachable, 1 skipped, 2 kept, 3 diagonal
    psum: np.ndarray       # [n][BM] fp64, sum of normalised probabilities over kept entries
    lse: np.ndarray        # [n][BM] fp32


def _pad_last_token(x: np.ndarray, n_pad: int) -> np.ndarray:
    """Section 4.3: a sequence that does not fill its last block is padded by repeating its
    last token."""
    N = x.shape[1]
    if n_pad == N:
        return x
    return np.ascontiguousarray(np.concatenate([x, np.repeat(x[:, N - 1:N], n_pad - N, axis=1)], axis=1))


def _expand_tau(tau, Hq, mq_pad):
    """Thresholds as the C oracle wants them.  Per-tile thresholds [Hq, T] with fewer tiles than
    the sequence has are extended with their last column: positions beyond the calibrated
    length reuse the thresholds of the last calibrated position (Section 4.3)."""
    tau = np.asarray(tau, dtype=np.float32)
    if tau.ndim == 1:
        assert tau.shape == (Hq,)
        return np.ascontiguousarray(tau), 0
    assert tau.ndim == 2 and tau.shape[0] == Hq and tau.shape[1] >= 1
    T = tau.shape[1]
    if T < mq_pad:
        tau = np.concatenate([tau, np.repeat(tau[:, T - 1:T], mq_pad - T, axis=1)], axis=1)
    return np.ascontiguousarray(tau[:, :mq_pad]), 1


def forward_items(q, k, v, tau, block_m, block_n, causal=True, items=None, forced_keep=None) -> ItemResult:
    """Evaluate the oracle on a list of (b, h, i) query tiles (all of them if ``items`` is None).

    q [B,N,Hq,d], k/v [B,N,Hkv,d]; tau [Hq] or [Hq, T] (T < M_Q: the last column serves every
    later tile); forced_keep optional [n_items, M_KV] overriding the gate on gateable blocks.
    M_Q = ceil(N / block_m), M_KV = ceil(N / block_n).  If N does not fill its last block
    (causal only) the inputs are padded by repeating the last token (Section 4.3), the padded
    problem is evaluated, and everything that belongs to padded rows or to key blocks made
    of padding only is dropped: rows >= N of the last tile come back as NaN."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    B, N, Hq, d = q.shape
    Hkv = k.shape[2]
    assert k.shape == (B, N, Hkv, d) and v.shape == k.shape
    MQ, MKV = -(-N // block_m), -(-N // block_n)
    big = max(block_m, block_n)
    assert big % block_m == 0 and big % block_n == 0
    n_pad = -(-N // big) * big
    if n_pad != N:
        assert causal, "padding by repetition is defined for the causal case only"
        q, k, v = (_pad_last_token(x, n_pad) for x in (q, k, v))
    mq_pad, mkv_pad = n_pad // block_m, n_pad // block_n
    tau, per_tile = _expand_tau(tau, Hq, mq_pad)
    if items is None:
        items = [(b, h, i) for b in range(B) for h in range(Hq) for i in range(MQ)]
    items = np.ascontiguousarray(np.asarray(items, dtype=np.int32).reshape(-1, 3))
    assert items[:, 2].max(initial=0) < MQ
    n = items.shape[0]
    fk = None
    if forced_keep is not None:
        fk = np.asarray(forced_keep, dtype=np.uint8)
        assert fk.shape == (n, MKV)
        fk = np.ascontiguousarray(np.pad(fk, ((0, 0), (0, mkv_pad - MKV)), constant_values=1))
    out = np.empty((n, block_m, d), np.float32)
    bmax = np.empty((n, mkv_pad), np.float32)
    cls = np.empty((n, mkv_pad), np.uint8)
    psum = np.empty((n, block_m), np.float64)
    lse = np.empty((n, block_m), np.float32)
    rc = _load().bsfa_oracle_items(
        _ptr(q, ctypes.c_float), _ptr(k, ctypes.c_float), _ptr(v, ctypes.c_float),
        B, n_pad, Hq, Hkv, d, block_m, block_n, int(bool(causal)),
        _ptr(tau, ctypes.c_float), per_tile, _ptr(items, ctypes.c_int32), n,
        _ptr(fk, ctypes.c_uint8), _ptr(out, ctypes.c_float), _ptr(bmax, ctypes.c_float),
        _ptr(cls, ctypes.c_uint8), _ptr(psum, ctypes.c_double), _ptr(lse, ctypes.c_float))
    if rc != 0:
        raise RuntimeError("bsfa_oracle_items failed with code %d" % rc)
    if n_pad != N:
        pad_rows = (items[:, 2:3] * block_m + np.arange(block_m)[None, :]) >= N     # [n, BM]
        out[pad_rows] = np.nan
        psum[pad_rows] = np.nan
        lse[pad_rows] = np.nan
        bmax = np.ascontiguousarray(bmax[:, :MKV])
        cls = np.ascontiguousarray(cls[:, :MKV])
    return ItemResult(items, out, bmax, cls, psum, lse)


@dataclass
class FullResult:
    out: np.ndarray        # [B,N,Hq,d] fp32
    bmax: np.ndarray       # [B,Hq,M_Q,M_KV] fp32 (NaN where not gateable)
    cls: np.ndarray        # [B,Hq,M_Q,M_KV] uint8
    psum: np.ndarray       # [B,N,Hq] fp64
    lse: np.ndarray        # [B,N,Hq] fp32
    counts: np.ndarray     # [B,Hq,3] int64: skipped, gateable, causally reachable tiles


def forward(q, k, v, tau, block_m, block_n, causal=True, forced_keep=None) -> FullResult:
    """Oracle on the whole problem, results re-assembled into tensor layout.
    ``forced_keep`` optional [B,Hq,M_Q,M_KV]; M_Q, M_KV rounded up for ragged N."""
    B, N, Hq, d = q.shape
    MQ, MKV = -(-N // block_m), -(-N // block_n)
    fk = None if forced_keep is None else np.asarray(forced_keep).reshape(B * Hq * MQ, MKV)
    r = forward_items(q, k, v, tau, block_m, block_n, causal, None, fk)
    out = r.out.reshape(B, Hq, MQ, block_m, d).transpose(0, 2, 3, 1, 4).reshape(B, MQ * block_m, Hq, d)[:, :N]
    psum = r.psum.reshape(B, Hq, MQ, block_m).transpose(0, 2, 3, 1).reshape(B, MQ * block_m, Hq)[:, :N]
    lse = r.lse.reshape(B, Hq, MQ, block_m).transpose(0, 2, 3, 1).reshape(B, MQ * block_m, Hq)[:, :N]
    cls = r.cls.reshape(B, Hq, MQ, MKV)
    return FullResult(np.ascontiguousarray(out), r.bmax.reshape(B, Hq, MQ, MKV), cls,
                      np.ascontiguousarray(psum), np.ascontiguousarray(lse), counts_from_cls(cls))


def counts_from_cls(cls: np.ndarray) -> np.ndarray:
    """Per (b, h): tiles skipped, tiles gateable, tiles reachable (measured density of
    Section 5.1's Metrics paragraph = 1 - skipped / reachable)."""
    skipped = (cls == CLS_SKIPPED).sum(axis=(-2, -1))
    gateable = ((cls == CLS_SKIPPED) | (cls == CLS_KEPT)).sum(axis=(-2, -1))
    reach = (cls != CLS_UNREACHABLE).sum(axis=(-2, -1))
    return np.stack([skipped, gateable, reach], axis=-1).astype(np.int64)


# --------------------------------------------------------------------------------------
# Algorithm 1, step by step (small inputs; numpy fp64)
# --------------------------------------------------------------------------------------
def alg1_tile(q, k, v, tau_h, b, h, i, block_m, block_n, order=None):
    """Algorithm 1 for one query block i of head h (causal), in the paper's notation.

    Gateable key blocks are visited in ``order`` (default ascending), each one gated on its
    block maximum; the blocks that touch the causal boundary follow, ungated, with the mask
    applied.  Returns (O_i [B_M, d], L_i [B_M], kept block indices)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, N, Hq, d = q.shape
    g = h // (Hq // k.shape[2])
    Qi = q[b, i * block_m:(i + 1) * block_m, h, :]
    m = np.full(block_m, -np.inf)
    l = np.zeros(block_m)
    O = np.zeros((block_m, d))
    n_reach = -(-((i + 1) * block_m) // block_n)
    gate = [j for j in range(n_reach) if (j + 1) * block_n - 1 <= i * block_m]
    diag = [j for j in range(n_reach) if j not in gate]
    if order is not None:
        assert sorted(order) == gate
        gate = list(order)
    kept = []

    def update(S, Vj):
        nonlocal m, l, O
        m_new = np.maximum(m, S.max(axis=1))
        P = np.exp(S - m_new[:, None])
        alpha = np.exp(m - m_new)
        O = O * alpha[:, None] + P @ Vj
        l = l * alpha + P.sum(axis=1)
        m = m_new

    for j in gate:
        Kj = k[b, j * block_n:(j + 1) * block_n, g, :]
        S = Qi @ Kj.T / np.sqrt(d)
        s_max = np.float32(S.max())
        if s_max >= np.float32(tau_h):            # skip iff s_max < T (Section 4.1)
            kept.append(j)
            update(S, v[b, j * block_n:(j + 1) * block_n, g, :])
    # diagonal blocks in ascending order: the first one gives every row a visible key, so
    # m stays finite in the later ones even where a whole row of S is masked
    for j in diag:
        Kj = k[b, j * block_n:(j + 1) * block_n, g, :]
        S = Qi @ Kj.T / np.sqrt(d)
        rows = i * block_m + np.arange(block_m)[:, None]
        cols = j * block_n + np.arange(block_n)[None, :]
        S = np.where(cols > rows, -np.inf, S)
        update(S, v[b, j * block_n:(j + 1) * block_n, g, :])
        kept.append(j)
    return O / l[:, None], m + np.log(l), kept


def alg1_tile_running_max(q, k, v, lam_h, b, h, i, block_m, block_n):
    """The comparison predicate of Section 3 (the in-kernel filter the paper describes for
    SpargeAttention) inside the loop of Algorithm 1, for one query block i of head h (causal,
    ascending block order, which the decisions now depend on).

    For a gateable block with score tile S_ij: m_local = row maxima of S_ij, m_ij = the running
    row maxima after the block, max(m_{i,j-1}, m_local), where m_{i,j-1} runs over the kept
    blocks before j (-inf before the first).  The block is skipped iff
    max over rows (m_local - m_ij) < lambda; skipped blocks leave (m, l, O) untouched.  The blocks
    that touch the causal boundary are processed ungated, as in Algorithm 1.
    Returns (O_i [B_M, d], L_i [B_M], kept block indices, statistic per gateable block as fp32)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, N, Hq, d = q.shape
    g = h // (Hq // k.shape[2])
    Qi = q[b, i * block_m:(i + 1) * block_m, h, :]
    m = np.full(block_m, -np.inf)
    l = np.zeros(block_m)
    O = np.zeros((block_m, d))
    n_reach = -(-((i + 1) * block_m) // block_n)
    kept, stats = [], {}
    for j in range(n_reach):
        Kj = k[b, j * block_n:(j + 1) * block_n, g, :]
        Vj = v[b, j * block_n:(j + 1) * block_n, g, :]
        S = Qi @ Kj.T / np.sqrt(d)
        gateable = (j + 1) * block_n - 1 <= i * block_m
        if gateable:
            m_local = S.max(axis=1)
            m_ij = np.maximum(m, m_local)
            stat = np.float32((m_local - m_ij).max())
            stats[j] = stat
            if stat < np.float32(lam_h):
                continue
        else:
            rows = i * block_m + np.arange(block_m)[:, None]
            cols = j * block_n + np.arange(block_n)[None, :]
            S = np.where(cols > rows, -np.inf, S)
        m_new = np.maximum(m, S.max(axis=1))
        P = np.exp(S - m_new[:, None])
        alpha = np.exp(m - m_new)
        O = O * alpha[:, None] + P @ Vj
        l = l * alpha + P.sum(axis=1)
        m = m_new
        kept.append(j)
    return O / l[:, None], m + np.log(l), kept, stats


# --------------------------------------------------------------------------------------
# Calibration
# --------------------------------------------------------------------------------------
def calibrate(bmax, cls_or_gateable, fractions) -> np.ndarray:
    """Per-head thresholds from block maxima of gateable tiles.

    bmax [B,Hq,M_Q,M_KV]; second argument either the class array or a boolean gateable mask.
    For a target skip fraction f over the n gateable tiles of a head (all batches pooled):
    sort ascending x_0 <= ... <= x_{n-1}; r = floor(f*n); tau = -inf if r == 0, +inf if r == n,
    else x_r.  With the keep rule s_max >= tau exactly r tiles are skipped (absent ties).
    Returns [n_levels, Hq] fp32."""
    bmax = np.asarray(bmax)
    a = np.asarray(cls_or_gateable)
    gate = a if a.dtype == bool else ((a == CLS_SKIPPED) | (a == CLS_KEPT))
    Hq = bmax.shape[1]
    out = np.empty((len(fractions), Hq), np.float32)
    for h in range(Hq):
        x = np.sort(bmax[:, h][gate[:, h]].astype(np.float32))
        n = x.size
        for li, f in enumerate(fractions):
            r = int(np.floor(np.float64(f) * n))
            out[li, h] = -np.inf if r <= 0 else (np.inf if r >= n else x[r])
    return out


def calibrate_topk(bmax_samples, gateable, ks) -> np.ndarray:
    """Section 4.2's rule: for each query tile, the threshold that retains exactly the top-k
    gateable blocks (the k-th largest block maximum; -inf when the tile has at most k gateable
    blocks, which keeps min(k, A) of them), averaged over calibration samples.

    bmax_samples: list of [Hq, M_Q, M_KV] arrays (one per calibration sample), gateable
    [M_Q, M_KV] bool.  Returns [n_levels, Hq, M_Q] fp32.  Tiles whose average would mix -inf
    with finite values stay -inf (cannot happen: availability depends on the tile only)."""
    gateable = np.asarray(gateable, dtype=bool)
    Hq, MQ, _ = np.asarray(bmax_samples[0]).shape
    acc = np.zeros((len(ks), Hq, MQ), np.float64)
    for bm in bmax_samples:
        bm = np.asarray(bm)
        for i in range(MQ):
            cols = np.nonzero(gateable[i])[0]
            A = cols.size
            for h in range(Hq):
                x = np.sort(bm[h, i, cols].astype(np.float32))[::-1]    # descending
                for li, kk in enumerate(ks):
                    acc[li, h, i] += -np.inf if A <= kk else x[kk - 1] if kk > 0 else np.inf
    return (acc / len(bmax_samples)).astype(np.float32)


def gateable_mask(seqlen, block_m, block_n, causal=True) -> np.ndarray:
    """[M_Q, M_KV] bool: blocks the gate applies to (fully visible, not overlapping the tile)."""
    MQ, MKV = -(-seqlen // block_m), -(-seqlen // block_n)
    i = np.arange(MQ)[:, None]
    j = np.arange(MKV)[None, :]
    if causal:
        return (j + 1) * block_n - 1 <= i * block_m
    return ~((j * block_n <= (i + 1) * block_m - 1) & ((j + 1) * block_n - 1 >= i * block_m))


def predicted_density(seqlen, block_m, block_n, k) -> float:
    """Section 5.1 (Metrics): (min(k, A) off-diagonal + diagonal blocks) / causally reachable
    blocks, A = gateable blocks of the query tile, summed over query tiles."""
    gate = gateable_mask(seqlen, block_m, block_n)
    MQ, MKV = gate.shape
    i = np.arange(MQ)[:, None]
    j = np.arange(MKV)[None, :]
    reach = j * block_n <= (i + 1) * block_m - 1
    A = gate.sum(axis=1)
    diag = reach.sum(axis=1) - A
    return float((np.minimum(k, A) + diag).sum() / reach.sum())
