"""CPU oracle for ASA with global tokens (ASA_G) -- TEST INFRASTRUCTURE ONLY.

Sec. 3.3, "ASA with Global Tokens": K and V are extended by mean-pooled copies of themselves
(windows of n tokens); a query sees the original keys through the binary block mask and ALL
pooled keys with ln(n) added to the pre-soft-max score.  Written out as that definition in
numpy fp64, one slab ``[L, d]`` at a time; no blocking beyond the block mask itself.

Readings where the paper is silent (listed in the design notes):
  * the pooled tokens are materialised in the model's tensor type: each element is the mean of
    the window's valid tokens rounded to bf16 (round to nearest even); `exact_pool=True` keeps
    the unrounded mean (used by the finite-difference pin, which needs a smooth function);
  * the last window may be short; its mean is over its valid tokens and its bias is ln(n) like
    every other window's ("a fixed additive mask of ln(n)");
  * the gradient flows through the pooling as through a plain mean (1 / count per token).

Parity against the authors' implementation is UNPINNED (no numeric example is printed); the pins
are in tests/test_oracle_global.py.
"""

from __future__ import annotations

import math
from typing import Optional, Sequence, Tuple

import numpy as np


def default_scale(d: int) -> float:
    """1/sqrt(d) as an fp32 value, the scale every entry point defaults to."""
    return float(np.float32(1.0) / np.sqrt(np.float32(d)))


def _round_bf16(x: np.ndarray) -> np.ndarray:
    """fp64 -> nearest bf16 (ties to even), returned as fp64."""
    f = np.ascontiguousarray(x, dtype=np.float32)        # bf16 means of bf16 data fit fp32 exactly enough:
    bits = f.view(np.uint32).astype(np.uint64)           # the second rounding acts on a 24-bit value
    lsb = (bits >> 16) & 1
    bits = (bits + 0x7FFF + lsb) >> 16 << 16
    return bits.astype(np.uint32).view(np.float32).astype(np.float64)


def n_windows(L: int, n: int) -> int:
    return (L + n - 1) // n


def pool(x: np.ndarray, n: int, exact_pool: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """MeanPool_n over the token axis of one slab [L, d] -> ([Lg, d] fp64, counts [Lg])."""
    L, d = x.shape
    Lg = n_windows(L, n)
    out = np.zeros((Lg, d), np.float64)
    cnt = np.zeros(Lg, np.int64)
    for w in range(Lg):
        rows = x[w * n:min(L, (w + 1) * n)].astype(np.float64)
        cnt[w] = rows.shape[0]
        out[w] = rows.sum(axis=0) / rows.shape[0]
    return (out if exact_pool else _round_bf16(out)), cnt


def _token_mask(mask: np.ndarray, L: int, b: int, rows: np.ndarray) -> np.ndarray:
    """Block mask [Nb, Nb] -> boolean [len(rows), L] for the given query tokens."""
    cols = np.arange(L) // b
    return mask[(rows // b)[:, None], cols[None, :]].astype(bool)


def attn_fwd_g(q, k, v, mask, b: int, n: int, scale: Optional[float] = None,
               qblocks: Optional[Sequence[int]] = None, exact_pool: bool = False):
    """O [L, d] fp64 and LSE [L] (natural log) of one slab; rows of unlisted query blocks are NaN."""
    L, d = q.shape
    scale = default_scale(d) if scale is None else scale
    kg, _ = pool(k, n, exact_pool)
    vg, _ = pool(v, n, exact_pool)
    Nb = (L + b - 1) // b
    blocks = range(Nb) if qblocks is None else qblocks
    o = np.full((L, d), np.nan)
    lse = np.full(L, np.nan)
    k64, v64 = k.astype(np.float64), v.astype(np.float64)
    for i in blocks:
        rows = np.arange(i * b, min(L, (i + 1) * b))
        qi = q[rows].astype(np.float64)
        s = scale * (qi @ k64.T)
        s[~_token_mask(mask, L, b, rows)] = -np.inf
        sg = scale * (qi @ kg.T) + math.log(n)
        sa = np.concatenate([s, sg], axis=1)
        m = sa.max(axis=1, keepdims=True)
        e = np.exp(sa - m)
        z = e.sum(axis=1, keepdims=True)
        p = e / z
        o[rows] = p[:, :L] @ v64 + p[:, L:] @ vg
        lse[rows] = (m + np.log(z))[:, 0]
    return o, lse


def attn_bwd_g(q, k, v, d_o, mask, b: int, n: int, scale: Optional[float] = None,
               exact_pool: bool = False):
    """dQ, dK, dV [L, d] fp64 of one slab (all query blocks), mask held constant."""
    L, d = q.shape
    scale = default_scale(d) if scale is None else scale
    kg, cnt = pool(k, n, exact_pool)
    vg, _ = pool(v, n, exact_pool)
    Lg = kg.shape[0]
    q64, k64, v64, g64 = (x.astype(np.float64) for x in (q, k, v, d_o))
    dq = np.zeros((L, d))
    dk = np.zeros((L, d))
    dv = np.zeros((L, d))
    dkg = np.zeros((Lg, d))
    dvg = np.zeros((Lg, d))
    Nb = (L + b - 1) // b
    for i in range(Nb):
        rows = np.arange(i * b, min(L, (i + 1) * b))
        qi, gi = q64[rows], g64[rows]
        s = scale * (qi @ k64.T)
        s[~_token_mask(mask, L, b, rows)] = -np.inf
        sa = np.concatenate([s, scale * (qi @ kg.T) + math.log(n)], axis=1)
        m = sa.max(axis=1, keepdims=True)
        e = np.exp(sa - m)
        p = e / e.sum(axis=1, keepdims=True)
        o_i = p[:, :L] @ v64 + p[:, L:] @ vg
        dp = np.concatenate([gi @ v64.T, gi @ vg.T], axis=1)
        delta = (gi * o_i).sum(axis=1, keepdims=True)
        ds = p * (dp - delta)
        dq[rows] = scale * (ds[:, :L] @ k64 + ds[:, L:] @ kg)
        dk += scale * (ds[:, :L].T @ qi)
        dv += p[:, :L].T @ gi
        dkg += scale * (ds[:, L:].T @ qi)
        dvg += p[:, L:].T @ gi
    win = np.arange(L) // n
    dk += dkg[win] / cnt[win][:, None]
    dv += dvg[win] / cnt[win][:, None]
    return dq, dk, dv
