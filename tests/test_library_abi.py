"""The C-ABI library loads and exports every symbol that include/asa.h declares (no GPU)."""

import ctypes
import os
import re

import pytest

from paper_2508_10774_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(headers=("asa.h", "asa_bench.h")):
    names = set()
    for h in headers:
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(asa_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_entry_points():
    names = _declared()
    for must in ("asa_build_mask", "asa_attn_fwd", "asa_attn_bwd", "asa_csr_from_mask",
                 "asa_mask_from_scores"):
        assert must in names
    assert sorted(binding.EXPORTS) == names
    # benchmark / test tooling is declared apart from the product interface
    product = _declared(("asa.h",))
    for tool in ("asa_mfma_rate_probe", "asa_set_kernel_timing", "asa_test_force_fwd_kernel"):
        assert tool not in product and tool in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2508_10774_amd import build
        build.build_lib()
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name
    assert binding.asa_version() == 100
    assert binding.load().asa_error_string(-1) == b"invalid argument"


def test_argument_errors_are_reported_without_a_gpu():
    # these calls fail validation before any HIP call is made
    L = binding.load()
    p = binding.Params(B=1, H=2, L=1024, d=96, block=64)
    assert L.asa_fwd_workspace_bytes(ctypes.byref(p.c())) == 0
    rc = L.asa_attn_fwd(ctypes.byref(p.c()), *([None] * 9), 0, None)
    assert rc == -2                                  # d = 96 is not built
    p = binding.Params(B=1, H=2, L=1024, d=64, block=64)
    assert L.asa_attn_fwd(ctypes.byref(p.c()), *([None] * 9), 0, None) == -1   # null pointers
    # V as transposed tiles, then the order of the forward's workgroups (256-byte granules)
    assert L.asa_fwd_workspace_bytes(ctypes.byref(p.c())) == 2 * 64 * 1024 * 2 + 256
    assert L.asa_attn_bwd(ctypes.byref(p.c()), *([None] * 15), 0, None) == -1
    assert L.asa_build_mask(ctypes.byref(p.c()), *([None] * 9), 0, None) == -1
    assert L.asa_mask_from_scores(ctypes.byref(p.c()), None, None, None) == -1
    # three fp32 row-statistics arrays [slab][Lpad] and the two workgroup orders (256-byte granules)
    assert L.asa_bwd_workspace_bytes(ctypes.byref(p.c())) == 3 * 2 * 1024 * 4 + 2 * 256
    # index lists: both (forward) / all four (backward) or none (dense); anything else is refused
    # before the pointers are looked at (the addresses below are never dereferenced)
    fake = ctypes.c_void_p(0x10000)
    assert L.asa_attn_fwd(ctypes.byref(p.c()), fake, fake, fake, fake, None, fake, None, fake,
                          fake, 1 << 30, None) == -1
    assert L.asa_attn_fwd(ctypes.byref(p.c()), fake, fake, fake, None, fake, fake, None, fake,
                          fake, 1 << 30, None) == -1
    assert L.asa_attn_bwd(ctypes.byref(p.c()), fake, fake, fake, fake, None, fake, fake,
                          fake, fake, fake, None, fake, fake, fake, fake, 1 << 30, None) == -1
    for bad in (dict(k_samples=0), dict(k_samples=65), dict(sample_offsets=[3, 1] + list(range(4, 18))),
                dict(r_min=0.6, r_max=0.5), dict(tau=float("nan")), dict(n_prefix_dense=-1),
                dict(q_stride=(0, 0, 60)), dict(k_stride=(1 << 40, 1 << 36, 1 << 24))):
        kw = dict(B=1, H=2, L=1024, d=64, block=64)
        kw.update(bad)
        pb = binding.Params(**kw)
        assert L.asa_mask_workspace_bytes(ctypes.byref(pb.c())) == 0, bad
    pb = binding.Params(B=1, H=1, L=64, d=64, block=32)
    assert L.asa_csr_from_mask(ctypes.byref(pb.c()), None, None, None, None, None, None) == -2
    with pytest.raises(binding.AsaError, match="unsupported"):
        binding._check(-2, "asa_csr_from_mask")
