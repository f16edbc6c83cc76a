"""asa_attn_bwd_noalloc (scratch memory in the library's own device array) against asa_attn_bwd
(scratch memory in a caller's workspace): same kernels, so the gradients must agree bit for bit.
Two calls in a row, the second on a smaller problem, so that the second finds the first one's
leftovers in the shared array."""

import numpy as np
import pytest
import torch

from paper_2508_10774_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu


def _case(B, H, L, d, block, dens, seed, with_lo):
    p = binding.Params(B=B, H=H, L=L, d=d, block=block)
    assert binding.asa_bwd_workspace_bytes(p) <= binding.NOALLOC_SCRATCH_BYTES
    shape = (B, H, L, d)
    q, k, v, g = (util.dev_bf16(synth.make_iid(shape, seed, s)) for s in range(4))
    mask = synth.random_block_mask(p.Nb, dens, seed=seed, slabs=B * H)
    bufs = util.lists_from_mask(p, mask)
    o, lse, o_lo = util.run_fwd(p, q, k, v, bufs, with_lo=True)
    if not with_lo:
        o_lo = None
    want = util.run_bwd(p, q, k, v, o, lse, g, bufs, o_lo=o_lo)
    return p, (q, k, v, o, g, lse, bufs, o_lo), want


def _run_noalloc(p, args):
    q, k, v, o, g, lse, bufs, o_lo = args
    dq = torch.full_like(q, float("nan"))
    dk = torch.full_like(k, float("nan"))
    dv = torch.full_like(v, float("nan"))
    binding.asa_attn_bwd_noalloc(p, q, k, v, o, g, lse, bufs["row_ptr"], bufs["col_idx"],
                                 bufs["col_ptr"], bufs["row_idx"], dq, dk, dv, o_lo=o_lo)
    torch.cuda.synchronize()
    return dq, dk, dv


def test_noalloc_backward_matches_the_workspace_backward_twice_in_a_row():
    print("case 1: B=1 H=3 L=2000 d=128 block=128", flush=True)
    p1, a1, want1 = _case(1, 3, 2000, 128, 128, 0.5, seed=31, with_lo=True)
    print("case 2: B=2 H=1 L=333 d=64 block=64 (smaller, no o_lo)", flush=True)
    p2, a2, want2 = _case(2, 1, 333, 64, 64, 0.6, seed=32, with_lo=False)
    got1 = _run_noalloc(p1, a1)
    got2 = _run_noalloc(p2, a2)      # finds case 1's row statistics and order in the array
    for got, want in ((got1, want1), (got2, want2)):
        for a, b, name in zip(got, want, ("dQ", "dK", "dV")):
            assert torch.isfinite(a.float()).all(), name
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), name


def test_noalloc_backward_refuses_what_does_not_fit():
    # 12 bytes per padded row: 960 000 rows need more than the 8 MiB array; refused before any launch
    p = binding.Params(B=1, H=8, L=120000, d=64, block=128)
    assert binding.asa_bwd_workspace_bytes(p) > binding.NOALLOC_SCRATCH_BYTES
    t = torch.zeros(64, dtype=torch.bfloat16, device="cuda")     # never touched
    f = torch.zeros(16, dtype=torch.float32, device="cuda")
    with pytest.raises(binding.AsaError, match="scratch"):
        binding.asa_attn_bwd_noalloc(p, t, t, t, t, t, f, None, None, None, None, t, t, t)
    torch.cuda.synchronize()
