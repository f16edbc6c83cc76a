"""ctypes binding of libasa.so: same entry-point names as ``include/asa.h``.

Argument marshalling only.  Tensors are torch CUDA(ROCm) tensors used for device memory
and streams; every step of the method runs in the HIP kernels of the library.  There is no
CPU or PyTorch fallback: if the library is missing or a call fails, an exception is raised.
"""

from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libasa.so")
_lib = None


class AsaError(RuntimeError):
    pass


class asa_params(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("L", ctypes.c_int32), ("d", ctypes.c_int32),
        ("block", ctypes.c_int32), ("k_samples", ctypes.c_int32),
        ("sample_offsets", ctypes.POINTER(ctypes.c_int32)),
        ("tau", ctypes.c_float), ("r_min", ctypes.c_float), ("r_max", ctypes.c_float),
        ("n_prefix_dense", ctypes.c_int32), ("scale", ctypes.c_float),
        ("q_stride", ctypes.c_int64 * 3), ("k_stride", ctypes.c_int64 * 3),
        ("v_stride", ctypes.c_int64 * 3), ("o_stride", ctypes.c_int64 * 3),
    ]


EXPORTS = ["asa_version", "asa_error_string", "asa_last_hip_error", "asa_mask_workspace_bytes",
           "asa_fwd_workspace_bytes", "asa_bwd_workspace_bytes", "asa_build_mask",
           "asa_mask_from_scores", "asa_csr_from_mask", "asa_attn_fwd", "asa_attn_bwd",
           "asa_attn_bwd_noalloc", "asa_set_kernel_timing", "asa_global_token_count", "asa_global_tokens",
           "asa_fwd_g_workspace_bytes", "asa_attn_fwd_g", "asa_bwd_g_workspace_bytes",
           "asa_attn_bwd_g", "asa_mask_seeded_workspace_bytes", "asa_build_mask_seeded",
           "asa_sample_offsets", "asa_gilbert_order", "asa_reorder_tokens",
           "asa_mfma_rate_probe", "asa_test_force_fwd_kernel", "asa_add_rate_probe"]


def load():
    """Load libasa.so (built by ``python -m paper_2508_10774_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise AsaError(f"{LIB_PATH} not found: build it with `python -m paper_2508_10774_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, pp = ctypes.c_void_p, ctypes.POINTER(asa_params)
    L.asa_version.restype = ctypes.c_int
    L.asa_error_string.restype = ctypes.c_char_p
    L.asa_error_string.argtypes = [ctypes.c_int]
    L.asa_last_hip_error.restype = ctypes.c_char_p
    for n in ("asa_mask_workspace_bytes", "asa_fwd_workspace_bytes", "asa_bwd_workspace_bytes",
              "asa_mask_seeded_workspace_bytes"):
        getattr(L, n).restype = ctypes.c_size_t
        getattr(L, n).argtypes = [pp]
    L.asa_build_mask.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.asa_build_mask_seeded.argtypes = [pp, ctypes.c_uint64] + [vp] * 9 + [ctypes.c_size_t, vp]
    L.asa_sample_offsets.argtypes = [pp, ctypes.c_uint64, vp, vp]
    L.asa_mask_from_scores.argtypes = [pp, vp, vp, vp]
    L.asa_csr_from_mask.argtypes = [pp, vp, vp, vp, vp, vp, vp]
    L.asa_attn_fwd.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.asa_attn_bwd.argtypes = [pp] + [vp] * 15 + [ctypes.c_size_t, vp]
    L.asa_attn_bwd_noalloc.argtypes = [pp] + [vp] * 15
    L.asa_attn_bwd_noalloc.restype = ctypes.c_int
    L.asa_set_kernel_timing.argtypes = [vp, vp]
    L.asa_add_rate_probe.argtypes = [ctypes.c_int32] * 4 + [vp, ctypes.POINTER(ctypes.c_double), vp]
    L.asa_add_rate_probe.restype = ctypes.c_int
    L.asa_test_force_fwd_kernel.argtypes = [ctypes.c_int]
    L.asa_test_force_fwd_kernel.restype = ctypes.c_int
    for n in ("asa_global_token_count", "asa_fwd_g_workspace_bytes", "asa_bwd_g_workspace_bytes"):
        getattr(L, n).restype = ctypes.c_size_t
        getattr(L, n).argtypes = [pp, ctypes.c_int]
    L.asa_global_tokens.argtypes = [pp, ctypes.c_int, vp, vp, vp, vp, vp]
    L.asa_attn_fwd_g.argtypes = [pp, ctypes.c_int] + [vp] * 11 + [ctypes.c_size_t, vp]
    L.asa_attn_bwd_g.argtypes = [pp, ctypes.c_int] + [vp] * 17 + [ctypes.c_size_t, vp]
    L.asa_mfma_rate_probe.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp,
                                      ctypes.POINTER(ctypes.c_double), vp]
    L.asa_mfma_rate_probe.restype = ctypes.c_int
    L.asa_gilbert_order.argtypes = [ctypes.c_int32] * 4 + [vp, vp]
    L.asa_reorder_tokens.argtypes = [pp, ctypes.c_int32, vp, vp, vp, vp, vp, vp]
    for n in ("asa_gilbert_order", "asa_reorder_tokens", "asa_build_mask", "asa_mask_from_scores", "asa_csr_from_mask", "asa_attn_fwd",
              "asa_attn_bwd", "asa_set_kernel_timing", "asa_global_tokens", "asa_attn_fwd_g",
              "asa_attn_bwd_g", "asa_build_mask_seeded", "asa_sample_offsets"):
        getattr(L, n).restype = ctypes.c_int
    _lib = L
    return L


@dataclass
class Params:
    """Python mirror of ``asa_params``; ``c()`` builds the C struct (keeps offsets alive)."""
    B: int
    H: int
    L: int
    d: int
    block: int
    k_samples: int = 16
    sample_offsets: Optional[Sequence[int]] = None
    tau: float = 0.9
    r_min: float = 0.0
    r_max: float = 1.0
    n_prefix_dense: int = 0
    scale: float = 0.0
    q_stride: Sequence[int] = (0, 0, 0)
    k_stride: Sequence[int] = (0, 0, 0)
    v_stride: Sequence[int] = (0, 0, 0)
    o_stride: Sequence[int] = (0, 0, 0)

    @property
    def Nb(self) -> int:
        return (self.L + self.block - 1) // self.block

    def c(self) -> asa_params:
        p = asa_params()
        p.B, p.H, p.L, p.d, p.block, p.k_samples = self.B, self.H, self.L, self.d, self.block, self.k_samples
        if self.sample_offsets is not None:
            arr = (ctypes.c_int32 * len(self.sample_offsets))(*[int(x) for x in self.sample_offsets])
            p._keep = arr
            p.sample_offsets = ctypes.cast(arr, ctypes.POINTER(ctypes.c_int32))
        p.tau, p.r_min, p.r_max = self.tau, self.r_min, self.r_max
        p.n_prefix_dense, p.scale = self.n_prefix_dense, self.scale
        for name in ("q_stride", "k_stride", "v_stride", "o_stride"):
            setattr(p, name, (ctypes.c_int64 * 3)(*[int(x) for x in getattr(self, name)]))
        return p


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise AsaError("libasa takes device tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _check(rc: int, what: str):
    if rc != 0:
        L = load()
        msg = L.asa_error_string(rc).decode()
        if rc == -4:
            msg += ": " + L.asa_last_hip_error().decode()
        raise AsaError(f"{what} failed ({rc}): {msg}")


def asa_version() -> int:
    return load().asa_version()


def asa_mask_workspace_bytes(p: Params) -> int:
    return load().asa_mask_workspace_bytes(ctypes.byref(p.c()))


def asa_fwd_workspace_bytes(p: Params) -> int:
    return load().asa_fwd_workspace_bytes(ctypes.byref(p.c()))


def asa_bwd_workspace_bytes(p: Params) -> int:
    return load().asa_bwd_workspace_bytes(ctypes.byref(p.c()))


def asa_build_mask(p: Params, q, k, mask, row_ptr, col_idx, col_ptr=None, row_idx=None,
                   p_imp=None, workspace=None, stream=None):
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load().asa_build_mask(ctypes.byref(p.c()), _ptr(q), _ptr(k), _ptr(mask), _ptr(row_ptr),
                               _ptr(col_idx), _ptr(col_ptr), _ptr(row_idx), _ptr(p_imp),
                               _ptr(workspace), ws_bytes, _stream(stream))
    _check(rc, "asa_build_mask")


def asa_mask_from_scores(p: Params, scores, mask, stream=None):
    _check(load().asa_mask_from_scores(ctypes.byref(p.c()), _ptr(scores), _ptr(mask),
                                       _stream(stream)), "asa_mask_from_scores")


def asa_csr_from_mask(p: Params, mask, row_ptr, col_idx, col_ptr=None, row_idx=None, stream=None):
    _check(load().asa_csr_from_mask(ctypes.byref(p.c()), _ptr(mask), _ptr(row_ptr), _ptr(col_idx),
                                    _ptr(col_ptr), _ptr(row_idx), _stream(stream)),
           "asa_csr_from_mask")


def asa_attn_fwd(p: Params, q, k, v, row_ptr, col_idx, o, lse, workspace, o_lo=None, stream=None):
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().asa_attn_fwd(ctypes.byref(p.c()), _ptr(q), _ptr(k), _ptr(v), _ptr(row_ptr),
                               _ptr(col_idx), _ptr(o), _ptr(o_lo), _ptr(lse), _ptr(workspace),
                               ws_bytes, _stream(stream)), "asa_attn_fwd")


def asa_attn_bwd(p: Params, q, k, v, o, d_o, lse, row_ptr, col_idx, col_ptr, row_idx, dq, dk, dv,
                 workspace, o_lo=None, stream=None):
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().asa_attn_bwd(ctypes.byref(p.c()), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(o_lo),
                               _ptr(d_o), _ptr(lse), _ptr(row_ptr), _ptr(col_idx), _ptr(col_ptr),
                               _ptr(row_idx), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(workspace),
                               ws_bytes, _stream(stream)), "asa_attn_bwd")


def asa_add_rate_probe(atomic: bool, workgroups: int, tiles_per_workgroup: int, n_qblocks: int, buf,
                       stream=None) -> float:
    """asa_bench.h: launches the calibration kernel; returns the payload bytes of the launch."""
    b = ctypes.c_double()
    _check(load().asa_add_rate_probe(int(bool(atomic)), workgroups, tiles_per_workgroup, n_qblocks,
                                     _ptr(buf), ctypes.byref(b), _stream(stream)), "asa_add_rate_probe")
    return b.value


def asa_test_force_fwd_kernel(which: int):
    """asa_bench.h: 0 = the library's choice, 1 = lock-step kernel, 2 = ping-pong kernel."""
    _check(load().asa_test_force_fwd_kernel(int(which)), "asa_test_force_fwd_kernel")


NOALLOC_SCRATCH_BYTES = 8 << 20   # ASA_NOALLOC_SCRATCH_BYTES of asa.h


def asa_attn_bwd_noalloc(p: Params, q, k, v, o, d_o, lse, row_ptr, col_idx, col_ptr, row_idx, dq,
                         dk, dv, o_lo=None, stream=None):
    _check(load().asa_attn_bwd_noalloc(ctypes.byref(p.c()), _ptr(q), _ptr(k), _ptr(v), _ptr(o),
                                       _ptr(o_lo), _ptr(d_o), _ptr(lse), _ptr(row_ptr),
                                       _ptr(col_idx), _ptr(col_ptr), _ptr(row_idx), _ptr(dq),
                                       _ptr(dk), _ptr(dv), _stream(stream)), "asa_attn_bwd_noalloc")


def asa_mask_seeded_workspace_bytes(p: Params) -> int:
    return int(load().asa_mask_seeded_workspace_bytes(ctypes.byref(p.c())))


def asa_build_mask_seeded(p: Params, seed: int, q, k, mask, row_ptr, col_idx, col_ptr, row_idx,
                          p_imp, workspace, stream=None):
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().asa_build_mask_seeded(ctypes.byref(p.c()), seed, _ptr(q), _ptr(k), _ptr(mask),
                                        _ptr(row_ptr), _ptr(col_idx), _ptr(col_ptr), _ptr(row_idx),
                                        _ptr(p_imp), _ptr(workspace), ws_bytes, _stream(stream)),
           "asa_build_mask_seeded")


def asa_sample_offsets(p: Params, seed: int, table, stream=None):
    _check(load().asa_sample_offsets(ctypes.byref(p.c()), seed, _ptr(table), _stream(stream)),
           "asa_sample_offsets")


def asa_global_token_count(p: Params, n: int) -> int:
    return int(load().asa_global_token_count(ctypes.byref(p.c()), n))


def asa_global_tokens(p: Params, n: int, k, v, kg, vg, stream=None):
    _check(load().asa_global_tokens(ctypes.byref(p.c()), n, _ptr(k), _ptr(v), _ptr(kg), _ptr(vg),
                                    _stream(stream)), "asa_global_tokens")


def asa_fwd_g_workspace_bytes(p: Params, n: int) -> int:
    return int(load().asa_fwd_g_workspace_bytes(ctypes.byref(p.c()), n))


def asa_attn_fwd_g(p: Params, n: int, q, k, v, kg, vg, row_ptr, col_idx, o, lse, workspace,
                   o_lo=None, stream=None):
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().asa_attn_fwd_g(ctypes.byref(p.c()), n, _ptr(q), _ptr(k), _ptr(v), _ptr(kg),
                                 _ptr(vg), _ptr(row_ptr), _ptr(col_idx), _ptr(o), _ptr(o_lo),
                                 _ptr(lse), _ptr(workspace), ws_bytes, _stream(stream)),
           "asa_attn_fwd_g")


def asa_bwd_g_workspace_bytes(p: Params, n: int) -> int:
    return int(load().asa_bwd_g_workspace_bytes(ctypes.byref(p.c()), n))


def asa_attn_bwd_g(p: Params, n: int, q, k, v, kg, vg, o, d_o, lse, row_ptr, col_idx, col_ptr,
                   row_idx, dq, dk, dv, workspace, o_lo=None, stream=None):
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().asa_attn_bwd_g(ctypes.byref(p.c()), n, _ptr(q), _ptr(k), _ptr(v), _ptr(kg),
                                 _ptr(vg), _ptr(o), _ptr(o_lo), _ptr(d_o), _ptr(lse), _ptr(row_ptr),
                                 _ptr(col_idx), _ptr(col_ptr), _ptr(row_idx), _ptr(dq), _ptr(dk),
                                 _ptr(dv), _ptr(workspace), ws_bytes, _stream(stream)),
           "asa_attn_bwd_g")


def asa_gilbert_order(T: int, Y: int, X: int, n_prefix: int = 0):
    """(order, inverse) as int32 CPU tensors of n_prefix + T*Y*X entries (host function)."""
    n = max(0, n_prefix) + max(0, T) * max(0, Y) * max(0, X)
    order = torch.empty(n, dtype=torch.int32)
    inverse = torch.empty(n, dtype=torch.int32)
    _check(load().asa_gilbert_order(T, Y, X, n_prefix, ctypes.c_void_p(order.data_ptr()),
                                    ctypes.c_void_p(inverse.data_ptr())), "asa_gilbert_order")
    return order, inverse


def asa_reorder_tokens(p: Params, src, dst, index, src_stride=None, dst_stride=None, stream=None):
    """dst[t][b, h, i, :] = src[t][b, h, index[i], :] for lists of up to three tensors."""
    n = len(src)
    if len(dst) != n:
        raise AsaError("asa_reorder_tokens: src and dst differ in length")
    srcs = (ctypes.c_void_p * n)(*[t.data_ptr() for t in src])
    dsts = (ctypes.c_void_p * n)(*[t.data_ptr() for t in dst])
    ss = (ctypes.c_int64 * 3)(*src_stride) if src_stride is not None else None
    ds = (ctypes.c_int64 * 3)(*dst_stride) if dst_stride is not None else None
    _check(load().asa_reorder_tokens(ctypes.byref(p.c()), n, srcs, dsts, ss, ds, _ptr(index),
                                     _stream(stream)), "asa_reorder_tokens")


def asa_mfma_rate_probe(workgroups: int, iters: int, sink, idle_sleep: int = 0, vector_stream: bool = False,
                        stream=None) -> float:
    """Launch the MFMA-only calibration kernel; returns the FLOP of the launch."""
    flop = ctypes.c_double(0.0)
    _check(load().asa_mfma_rate_probe(workgroups, iters, idle_sleep, int(vector_stream), _ptr(sink),
                                      ctypes.byref(flop), _stream(stream)), "asa_mfma_rate_probe")
    return flop.value


def asa_set_kernel_timing(start: Optional[torch.cuda.Event], stop: Optional[torch.cuda.Event]):
    """Arm the one-shot hook with two torch events (they must have been recorded once, which
    is what creates their HIP handles)."""
    a = ctypes.c_void_p(start.cuda_event) if start is not None else None
    b = ctypes.c_void_p(stop.cuda_event) if stop is not None else None
    _check(load().asa_set_kernel_timing(a, b), "asa_set_kernel_timing")


# ---------------------------------------------------------------------------
# device-memory helpers (allocation only)
# ---------------------------------------------------------------------------

def alloc_index_lists(p: Params, device="cuda", with_csc: bool = True):
    """Empty mask / CSR / CSC buffers of the sizes ``asa.h`` documents."""
    S, Nb = p.B * p.H, p.Nb
    out = {
        "mask": torch.empty((S, Nb, Nb), dtype=torch.uint8, device=device),
        "row_ptr": torch.empty((S, Nb + 1), dtype=torch.int32, device=device),
        "col_idx": torch.empty((S, Nb * Nb), dtype=torch.int32, device=device),
    }
    if with_csc:
        out["col_ptr"] = torch.empty((S, Nb + 1), dtype=torch.int32, device=device)
        out["row_idx"] = torch.empty((S, Nb * Nb), dtype=torch.int32, device=device)
    return out


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty((max(int(nbytes), 256),), dtype=torch.uint8, device=device)
