"""CPU oracle for Adaptive Block-Sparse Attention -- TEST INFRASTRUCTURE ONLY.

A thin ctypes layer over ``asa_ref.c`` (plain C, fp64 arithmetic) plus the
few numpy lines that loop over (batch, head) slabs and turn a mask into
CSR/CSC lists.  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product path never does,
and this package never imports the product path.

Inputs are fp32 numpy arrays whose values are exactly representable in bf16
(the bits the GPU sees, widened); one slab is ``[L, d]``.

Parity against the authors' implementation is UNPINNED (the paper prints no
numeric example).  The pins that stand in for it are in ``tests/test_oracle_*``.
"""

from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "asa_ref.c")
_LIB = os.path.join(_HERE, "libasa_ref.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile asa_ref.c with gcc; returns the path of the shared library."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        # (x86-64-v3, not native: the built library travels with the tree to other hosts)
        cmd = ["gcc", "-std=c11", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _c(arr, dtype):
    a = np.ascontiguousarray(arr, dtype=dtype)
    return a


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        up = ctypes.POINTER(ctypes.c_uint8)
        ci = ctypes.c_int
        L.asa_ref_num_threads.restype = ci
        L.asa_ref_sample_rows.argtypes = [ci, ci, ci, ip, ip]
        for name in ("asa_ref_p_imp_direct", "asa_ref_p_imp_online"):
            getattr(L, name).argtypes = [fp, fp, ci, ci, ci, ci, ip, ctypes.c_float, fp]
        L.asa_ref_retention_bounds.argtypes = [ci, ctypes.c_float, ctypes.c_float, ip, ip]
        for name in ("asa_ref_mask_rule_sort", "asa_ref_mask_rule_orderfree"):
            getattr(L, name).argtypes = [fp, ci, ci, ctypes.c_float, ci, ci, up, ip]
        L.asa_ref_force_prefix.argtypes = [up, ci, ci, ci]
        L.asa_ref_attn_fwd.argtypes = [fp, fp, fp, ci, ci, ci, up, ctypes.c_double, ip, ci, dp, dp]
        L.asa_ref_attn_delta.argtypes = [fp, dp, ci, ci, ci, ip, ci, dp]
        L.asa_ref_attn_bwd_dq.argtypes = [fp, fp, fp, fp, ci, ci, ci, up, ctypes.c_double, dp, dp,
                                          ip, ci, dp]
        L.asa_ref_attn_bwd_dkv.argtypes = [fp, fp, fp, fp, ci, ci, ci, up, ctypes.c_double, dp, dp,
                                           ip, ci, dp, dp]
        L.asa_ref_attn_bwd_dq_mag.argtypes = L.asa_ref_attn_bwd_dq.argtypes
        L.asa_ref_attn_bwd_dkv_mag.argtypes = L.asa_ref_attn_bwd_dkv.argtypes
        _lib = L
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def num_threads() -> int:
    return int(lib().asa_ref_num_threads())


def n_blocks(L: int, b: int) -> int:
    return (L + b - 1) // b


def default_scale(d: int) -> float:
    """1/sqrt(d) as an fp32 value (the softmax scale of Alg. 3 step 4)."""
    return float(np.float32(1.0) / np.sqrt(np.float32(d)))


# ---------------------------------------------------------------------------
# mask path
# ---------------------------------------------------------------------------

def sample_rows(L: int, b: int, offs: Sequence[int]) -> np.ndarray:
    """Token index of every (block, sample) pair, -1 where it falls in the padding."""
    offs = _c(offs, np.int32)
    out = np.empty(n_blocks(L, b) * len(offs), dtype=np.int32)
    _check(lib().asa_ref_sample_rows(L, b, len(offs), _p(offs, ctypes.c_int32),
                                     _p(out, ctypes.c_int32)), "sample_rows")
    return out


def p_imp(q: np.ndarray, k: np.ndarray, b: int, offs: Sequence[int],
          scale: Optional[float] = None, form: str = "direct") -> np.ndarray:
    """Block importance map [Nb, Nb] (fp32) of one slab; form = 'direct' | 'online'."""
    q = _c(q, np.float32)
    k = _c(k, np.float32)
    L, d = q.shape
    assert k.shape == (L, d)
    offs = _c(offs, np.int32)
    if scale is None:
        scale = default_scale(d)
    Nb = n_blocks(L, b)
    out = np.empty((Nb, Nb), dtype=np.float32)
    fn = {"direct": lib().asa_ref_p_imp_direct, "online": lib().asa_ref_p_imp_online}[form]
    _check(fn(_p(q, ctypes.c_float), _p(k, ctypes.c_float), L, d, b, len(offs),
              _p(offs, ctypes.c_int32), ctypes.c_float(scale), _p(out, ctypes.c_float)),
           "p_imp_" + form)
    return out


def retention_bounds(Nb: int, r_min: float, r_max: float) -> Tuple[int, int]:
    lo = ctypes.c_int32()
    hi = ctypes.c_int32()
    _check(lib().asa_ref_retention_bounds(Nb, ctypes.c_float(r_min), ctypes.c_float(r_max),
                                          ctypes.byref(lo), ctypes.byref(hi)), "retention_bounds")
    return lo.value, hi.value


def mask_rule(scores: np.ndarray, tau: float, r_min: float = 0.0, r_max: float = 1.0,
              form: str = "sort") -> Tuple[np.ndarray, np.ndarray]:
    """Apply the selection rule to rows of scores [..., Nb]; returns (mask u8, m int32)."""
    scores = _c(scores, np.float32)
    Nb = scores.shape[-1]
    rows = int(np.prod(scores.shape[:-1], dtype=np.int64))
    m_min, m_max = retention_bounds(Nb, r_min, r_max)
    mask = np.empty(scores.shape, dtype=np.uint8)
    m = np.empty(scores.shape[:-1], dtype=np.int32)
    fn = {"sort": lib().asa_ref_mask_rule_sort,
          "orderfree": lib().asa_ref_mask_rule_orderfree}[form]
    _check(fn(_p(scores, ctypes.c_float), rows, Nb, ctypes.c_float(tau), m_min, m_max,
              _p(mask, ctypes.c_uint8), _p(m, ctypes.c_int32)), "mask_rule_" + form)
    return mask, m


def force_prefix(mask: np.ndarray, b: int, n_prefix: int) -> np.ndarray:
    """OR the always-kept prefix rows/columns into masks [..., Nb, Nb] (in a copy)."""
    mask = np.array(mask, dtype=np.uint8, order="C", copy=True)
    Nb = mask.shape[-1]
    flat = mask.reshape(-1, Nb, Nb)
    for s in range(flat.shape[0]):
        sl = flat[s]
        _check(lib().asa_ref_force_prefix(_p(sl, ctypes.c_uint8), Nb, b, n_prefix), "force_prefix")
    return mask


def build_mask(q: np.ndarray, k: np.ndarray, b: int, offs: Sequence[int], tau: float,
               r_min: float = 0.0, r_max: float = 1.0, n_prefix: int = 0,
               scale: Optional[float] = None, form: str = "direct"):
    """Mask path for q, k of shape [B, H, L, d]: returns (mask [B,H,Nb,Nb] u8, p_imp fp32)."""
    B, H, L, d = q.shape
    Nb = n_blocks(L, b)
    P = np.empty((B, H, Nb, Nb), dtype=np.float32)
    for bi in range(B):
        for h in range(H):
            P[bi, h] = p_imp(q[bi, h], k[bi, h], b, offs, scale, form)
    mask, _ = mask_rule(P, tau, r_min, r_max)
    if n_prefix > 0:
        mask = force_prefix(mask, b, n_prefix)
    return mask, P


def csr_from_mask(mask: np.ndarray):
    """row_ptr [S, Nb+1], col_idx [S, Nb*Nb] (ascending in a row, -1 beyond nnz) per slab."""
    Nb = mask.shape[-1]
    flat = mask.reshape(-1, Nb, Nb)
    S = flat.shape[0]
    row_ptr = np.zeros((S, Nb + 1), dtype=np.int32)
    col_idx = np.full((S, Nb * Nb), -1, dtype=np.int32)
    for s in range(S):
        cnt = flat[s].astype(bool).sum(axis=1)
        row_ptr[s, 1:] = np.cumsum(cnt)
        r, c = np.nonzero(flat[s])
        col_idx[s, : len(c)] = c
    return row_ptr, col_idx


def csc_from_mask(mask: np.ndarray):
    """col_ptr [S, Nb+1], row_idx [S, Nb*Nb] (ascending in a column) per slab."""
    Nb = mask.shape[-1]
    flat = mask.reshape(-1, Nb, Nb)
    return csr_from_mask(np.ascontiguousarray(np.swapaxes(flat, 1, 2)))


# ---------------------------------------------------------------------------
# attention
# ---------------------------------------------------------------------------

def _blocks(arg, Nb):
    if arg is None:
        return np.arange(Nb, dtype=np.int32)
    return _c(np.asarray(arg).reshape(-1), np.int32)


def attn_fwd(q, k, v, mask, b: int, scale: Optional[float] = None, qblocks=None):
    """Masked attention of one slab.  Returns (O [L,d] f64, LSE [L] f64); rows outside
    the listed query blocks are NaN."""
    q = _c(q, np.float32); k = _c(k, np.float32); v = _c(v, np.float32)
    L, d = q.shape
    Nb = n_blocks(L, b)
    mask = _c(mask, np.uint8)
    assert mask.shape == (Nb, Nb)
    if scale is None:
        scale = default_scale(d)
    qb = _blocks(qblocks, Nb)
    o = np.full((L, d), np.nan, dtype=np.float64)
    lse = np.full((L,), np.nan, dtype=np.float64)
    _check(lib().asa_ref_attn_fwd(_p(q, ctypes.c_float), _p(k, ctypes.c_float),
                                  _p(v, ctypes.c_float), L, d, b, _p(mask, ctypes.c_uint8),
                                  ctypes.c_double(scale), _p(qb, ctypes.c_int32), len(qb),
                                  _p(o, ctypes.c_double), _p(lse, ctypes.c_double)), "attn_fwd")
    return o, lse


def attn_bwd(q, k, v, d_o, mask, b: int, scale: Optional[float] = None, qblocks=None,
             kblocks=None, with_mag: bool = False):
    """Gradients of one slab with the mask held constant.

    Returns (dQ, dK, dV) as [L, d] f64; dQ rows outside ``qblocks`` and dK/dV rows outside
    ``kblocks`` are NaN.  O, LSE and Delta are recomputed here in fp64 for exactly the
    query blocks the requested outputs depend on.

    with_mag: also return (dQ_mag, dK_mag, dV_mag), the sums of the absolute values of the
    terms that each gradient element adds up (what bounds the rounding error of a reduced-
    precision implementation; used by the tests' tolerance only).
    """
    q = _c(q, np.float32); k = _c(k, np.float32); v = _c(v, np.float32)
    d_o = _c(d_o, np.float32)
    L, d = q.shape
    Nb = n_blocks(L, b)
    mask = _c(mask, np.uint8)
    if scale is None:
        scale = default_scale(d)
    qb = _blocks(qblocks, Nb)
    kb = _blocks(kblocks, Nb)
    need = set(int(x) for x in qb)
    for j in kb:
        need.update(int(i) for i in np.nonzero(mask[:, j])[0])
    need = np.array(sorted(need), dtype=np.int32)
    o, lse = attn_fwd(q, k, v, mask, b, scale, need)
    delta = np.full((L,), np.nan, dtype=np.float64)
    _check(lib().asa_ref_attn_delta(_p(d_o, ctypes.c_float), _p(o, ctypes.c_double), L, d, b,
                                    _p(need, ctypes.c_int32), len(need),
                                    _p(delta, ctypes.c_double)), "attn_delta")
    dq = np.full((L, d), np.nan, dtype=np.float64)
    dk = np.full((L, d), np.nan, dtype=np.float64)
    dv = np.full((L, d), np.nan, dtype=np.float64)
    args = (_p(q, ctypes.c_float), _p(k, ctypes.c_float), _p(v, ctypes.c_float),
            _p(d_o, ctypes.c_float), L, d, b, _p(mask, ctypes.c_uint8), ctypes.c_double(scale),
            _p(lse, ctypes.c_double), _p(delta, ctypes.c_double))
    if len(qb):
        _check(lib().asa_ref_attn_bwd_dq(*args, _p(qb, ctypes.c_int32), len(qb),
                                         _p(dq, ctypes.c_double)), "attn_bwd_dq")
    if len(kb):
        _check(lib().asa_ref_attn_bwd_dkv(*args, _p(kb, ctypes.c_int32), len(kb),
                                          _p(dk, ctypes.c_double), _p(dv, ctypes.c_double)),
               "attn_bwd_dkv")
    if not with_mag:
        return dq, dk, dv
    mq = np.full((L, d), np.nan, dtype=np.float64)
    mk = np.full((L, d), np.nan, dtype=np.float64)
    mv = np.full((L, d), np.nan, dtype=np.float64)
    if len(qb):
        _check(lib().asa_ref_attn_bwd_dq_mag(*args, _p(qb, ctypes.c_int32), len(qb),
                                             _p(mq, ctypes.c_double)), "attn_bwd_dq_mag")
    if len(kb):
        _check(lib().asa_ref_attn_bwd_dkv_mag(*args, _p(kb, ctypes.c_int32), len(kb),
                                              _p(mk, ctypes.c_double), _p(mv, ctypes.c_double)),
               "attn_bwd_dkv_mag")
    return dq, dk, dv, mq, mk, mv
