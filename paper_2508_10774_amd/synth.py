"""Seeded synthetic video-token tensors for ASA tests and benchmarks.

This module only draws inputs.  It holds none of the method's arithmetic
(no sampling of representative tokens, no scores, no masks, no attention), so
that the CPU oracle and the HIP path can both be fed from it without sharing
any code of their own.

Recipe (stands in for DiT activations, which need the models' weights):

* ``V``  : iid N(0,1).
* ``Q,K``: iid N(0,1) plus a *shared* smooth field ``gain * S``.  ``S`` is
  white noise per head and per channel on the T x Y x X token grid, blurred
  with a separable Gaussian (sigma tokens per axis, truncated at 4 sigma,
  reflecting boundary) and re-scaled to unit standard deviation per head.
  Neighbouring tokens therefore share a direction in feature space, which is
  the locality prior the paper's Sec. 3.3 builds on.
* Tokens are flattened in raster order (t major, then y, then x).  Optional
  ``n_text`` iid N(0,1) tokens are placed before the grid (CogVideoX layout).
* Everything is rounded to bf16 (round-to-nearest-even) once, on the host;
  every consumer sees exactly those bits.

The four random streams (noise_Q, noise_K, V, smooth) come from
``numpy.random.SeedSequence(seed).spawn(4)``; a fifth, spawned from
``SeedSequence([seed, 1])``, gives ``dO`` for the training path.
"""

from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np


# --------------------------------------------------------------------------
# bf16 <-> fp32 bit helpers (storage format only)
# --------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 with round-to-nearest-even; returns uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    nan = np.isnan(x)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    r = r.astype(np.uint16)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen uint16 bf16 bits to fp32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 values that are exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    d: int
    grid: Tuple[int, int, int]   # (T, Y, X) video-token grid
    n_text: int                  # iid tokens placed before the grid
    block: int
    k_samples: int

    @property
    def L(self) -> int:
        t, y, x = self.grid
        return self.n_text + t * y * x

    @property
    def Nb(self) -> int:
        return (self.L + self.block - 1) // self.block


TINY = Workload("tiny", 1, 2, 64, (4, 16, 16), 0, 64, 16)
WAN = Workload("wan2.1-1.3b", 1, 12, 128, (21, 30, 52), 0, 128, 16)
WAN_PADDED = Workload("wan2.1-1.3b-L32768", 1, 12, 128, (32, 32, 32), 0, 128, 16)
COG = Workload("cogvideox-5b", 1, 48, 64, (13, 30, 45), 226, 64, 16)

WORKLOADS = {w.name: w for w in (TINY, WAN, WAN_PADDED, COG)}


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------

def _gauss_kernel(sigma: float) -> np.ndarray:
    r = int(4.0 * sigma + 0.5)
    t = np.arange(-r, r + 1, dtype=np.float64)
    w = np.exp(-0.5 * (t / sigma) ** 2)
    return (w / w.sum()).astype(np.float32)


def _blur_axis(a: np.ndarray, axis: int, sigma: float) -> np.ndarray:
    """Gaussian blur along one axis, reflecting boundary (d c b a | a b c d | d c b a)."""
    w = _gauss_kernel(sigma)
    r = (len(w) - 1) // 2
    n = a.shape[axis]
    # reflect-pad by index arithmetic so that short axes (n < r) also work
    idx = np.arange(-r, n + r)
    period = 2 * n
    idx = np.mod(idx, period)
    idx = np.where(idx >= n, period - 1 - idx, idx)
    ap = np.take(a, idx, axis=axis)
    out = np.zeros_like(a)
    sl = [slice(None)] * a.ndim
    for t in range(2 * r + 1):
        sl[axis] = slice(t, t + n)
        out += w[t] * ap[tuple(sl)]
    return out


def smooth_field(rng: np.random.Generator, H: int, grid: Tuple[int, int, int], d: int,
                 sigma: float = 2.0) -> np.ndarray:
    """[H, T*Y*X, d] fp32 field, unit standard deviation per head."""
    T, Y, X = grid
    s = rng.standard_normal((H, T, Y, X, d), dtype=np.float32)
    for ax in (1, 2, 3):
        s = _blur_axis(s, ax, sigma)
    s = s.reshape(H, T * Y * X, d)
    std = s.std(axis=(1, 2), keepdims=True, dtype=np.float64).astype(np.float32)
    s /= std
    return s


def make_qkv(w: Workload, seed: int, gain: float = 2.0, sigma: float = 2.0,
             restandardise: bool = True):
    """Return (q, k, v) as uint16 bf16 bit arrays of shape [B, H, L, d]."""
    ss = np.random.SeedSequence(seed).spawn(4)
    rq, rk, rv, rs = (np.random.default_rng(s) for s in ss)
    shape = (w.B, w.H, w.L, w.d)
    q = rq.standard_normal(shape, dtype=np.float32)
    k = rk.standard_normal(shape, dtype=np.float32)
    v = rv.standard_normal(shape, dtype=np.float32)
    for b in range(w.B):
        if restandardise:
            s = smooth_field(rs, w.H, w.grid, w.d, sigma)
        else:
            T, Y, X = w.grid
            s = rs.standard_normal((w.H, T, Y, X, w.d), dtype=np.float32)
            for ax in (1, 2, 3):
                s = _blur_axis(s, ax, sigma)
            s = s.reshape(w.H, T * Y * X, w.d)
        s *= np.float32(gain)
        q[b, :, w.n_text:, :] += s
        k[b, :, w.n_text:, :] += s
        del s
    return f32_to_bf16_bits(q), f32_to_bf16_bits(k), f32_to_bf16_bits(v)


def make_do(w: Workload, seed: int) -> np.ndarray:
    """Upstream gradient dO ~ N(0,1), bf16 bits [B, H, L, d]."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 1]))
    return f32_to_bf16_bits(rng.standard_normal((w.B, w.H, w.L, w.d), dtype=np.float32))


def make_iid(shape, seed: int, stream: int = 0) -> np.ndarray:
    """iid N(0,1) bf16 bits, for unit tests that need no grid structure."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 7, stream]))
    return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))


def random_block_mask(Nb: int, density: float, seed: int, slabs: int = 1) -> np.ndarray:
    """uint8 [slabs, Nb, Nb] random mask with >= 1 kept block per row (test input)."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 11]))
    m = (rng.random((slabs, Nb, Nb)) < density).astype(np.uint8)
    forced = rng.integers(0, Nb, size=(slabs, Nb))
    s_idx, r_idx = np.meshgrid(np.arange(slabs), np.arange(Nb), indexing="ij")
    m[s_idx, r_idx, forced] = 1
    return m


def default_sample_offsets(block: int, k: int) -> np.ndarray:
    """Deterministic strided offsets u * (block // k), the library's default."""
    return (np.arange(k, dtype=np.int32) * (block // k)).astype(np.int32)


def random_sample_offsets(block: int, k: int, seed: int) -> np.ndarray:
    """k distinct ascending offsets in [0, block), drawn by the caller (Alg. 3 step 3)."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 13]))
    return np.sort(rng.choice(block, size=k, replace=False)).astype(np.int32)
