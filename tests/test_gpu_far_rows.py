"""Key rows 2 MiB apart (a K slab of 4.4 GB): every kernel has to address K, and dK, with 64-bit
arithmetic, and the forward has to fall back from its 32-bit tile offsets.  Parity as elsewhere."""

import numpy as np
import pytest
import torch

import oracle
from paper_2508_10774_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu

L, D, BLOCK, ROW_PITCH = 2100, 128, 128, 1 << 20     # elements between consecutive key rows


def _far_rows(bits=None):
    storage = torch.empty((L - 1) * ROW_PITCH + D, dtype=torch.bfloat16, device="cuda")
    view = storage.as_strided((1, 1, L, D), (L * ROW_PITCH, L * ROW_PITCH, ROW_PITCH, 1))
    if bits is not None:
        view.copy_(util.dev_bf16(bits))
    return storage, view


def test_mask_forward_backward_with_key_rows_two_mebibytes_apart():
    stride = (L * ROW_PITCH, L * ROW_PITCH, ROW_PITCH)
    p = binding.Params(B=1, H=1, L=L, d=D, block=BLOCK, tau=0.9, k_stride=stride)
    assert p.Nb * BLOCK * ROW_PITCH * 2 >= 1 << 32
    shape = (1, 1, L, D)
    qb, kb, vb, gb = (synth.make_iid(shape, 77, s) for s in range(4))
    q, v, g = (util.dev_bf16(x) for x in (qb, vb, gb))
    k_store, k = _far_rows(kb)
    qf, kf, vf, gf = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb, gb))

    # mask
    bufs = binding.alloc_index_lists(p)
    p_imp = torch.empty((1, p.Nb, p.Nb), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(binding.asa_mask_workspace_bytes(p))
    binding.asa_build_mask(p, q, k, bufs["mask"], bufs["row_ptr"], bufs["col_idx"], bufs["col_ptr"],
                           bufs["row_idx"], p_imp, ws)
    torch.cuda.synchronize()
    offs = synth.default_sample_offsets(BLOCK, 16)
    mask_o, P = oracle.build_mask(qf, kf, BLOCK, offs, 0.9)
    np.testing.assert_allclose(p_imp.cpu().numpy()[0], P[0, 0], rtol=1e-4, atol=1e-30)
    mask_g = bufs["mask"].cpu().numpy().reshape(mask_o.shape)
    exact, excused, failed = util.classify_mask_rows(P, mask_o, mask_g, 0.9)
    assert not failed, failed

    # forward and backward on a denser random mask
    mask = synth.random_block_mask(p.Nb, 0.5, seed=3, slabs=1)
    bufs = util.lists_from_mask(p, mask)
    o, lse, o_lo = util.run_fwd(p, q, k, v, bufs, with_lo=True)
    want_o, want_lse = oracle.attn_fwd(qf[0, 0], kf[0, 0], vf[0, 0], mask[0], BLOCK)
    util.assert_close_bf16(util.host_f32(o)[0, 0], want_o, "O")
    assert np.abs(lse.cpu().numpy()[0] - want_lse).max() <= util.LSE_ABS

    dq, dv = torch.full_like(q, float("nan")), torch.full_like(v, float("nan"))
    dk_store, dk = _far_rows()
    wsb = binding.alloc_workspace(binding.asa_bwd_workspace_bytes(p))
    binding.asa_attn_bwd(p, q, k, v, o, g, lse, bufs["row_ptr"], bufs["col_idx"], bufs["col_ptr"],
                         bufs["row_idx"], dq, dk, dv, wsb, o_lo=o_lo)
    torch.cuda.synchronize()
    wq, wk, wv = oracle.attn_bwd(qf[0, 0], kf[0, 0], vf[0, 0], gf[0, 0], mask[0], BLOCK)
    util.assert_close_bf16(util.host_f32(dq)[0, 0], wq, "dQ")
    util.assert_close_bf16(util.host_f32(dk.contiguous())[0, 0], wk, "dK")
    util.assert_close_bf16(util.host_f32(dv)[0, 0], wv, "dV")

    # global tokens need contiguous key rows: refused before anything is launched
    n = 128
    G = binding.asa_global_token_count(p, n)
    kg = torch.empty((1, 1, G, D), dtype=torch.bfloat16, device="cuda")
    vg = torch.empty_like(kg)
    binding.asa_global_tokens(p, n, k, v, kg, vg)
    wsg = binding.alloc_workspace(binding.asa_fwd_g_workspace_bytes(p, n))
    with pytest.raises(binding.AsaError):
        binding.asa_attn_fwd_g(p, n, q, k, v, kg, vg, bufs["row_ptr"], bufs["col_idx"], o, lse, wsg)
    torch.cuda.synchronize()
    del k_store, dk_store
