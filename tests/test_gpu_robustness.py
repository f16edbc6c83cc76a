"""Properties that hold whatever the inputs: nothing outside the tensors is written (canary rows
around every output), and non-finite inputs still give a valid mask and valid index lists."""

import numpy as np
import pytest
import torch

from paper_2508_10774_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu

CANARY = 0x7FC5          # a bf16 NaN with a payload no kernel produces
GUARD_ROWS = 24


def _guarded(B, H, L, d):
    """A [B, H, L, d] bf16 view whose slabs are GUARD_ROWS + L + GUARD_ROWS rows apart: rows past L
    of a slab (where a kernel that wrote whole tiles would land) and rows before it are canaries."""
    rows = GUARD_ROWS + L + GUARD_ROWS
    store = torch.full((B * H * rows * d + 2 * GUARD_ROWS * d,), CANARY, dtype=torch.int16, device="cuda")
    body = store[GUARD_ROWS * d:GUARD_ROWS * d + B * H * rows * d].view(B, H, rows, d)
    view = body[:, :, GUARD_ROWS:GUARD_ROWS + L, :].view(torch.bfloat16)
    stride = (H * rows * d, rows * d, d)
    return store, view, stride


def _canaries_intact(store, view, what):
    probe = store.clone()
    B, H, L, d = view.shape
    rows = GUARD_ROWS + L + GUARD_ROWS
    body = probe[GUARD_ROWS * d:GUARD_ROWS * d + B * H * rows * d].view(B, H, rows, d)
    body[:, :, GUARD_ROWS:GUARD_ROWS + L, :] = CANARY       # blank the tensor itself
    assert bool((probe == CANARY).all()), f"{what}: a row outside the tensor was written"
    assert bool((view.view(torch.int16) != CANARY).all()), f"{what}: a row of the tensor was not written"


@pytest.mark.parametrize("L,d,block", [(1000, 128, 128), (333, 64, 64), (450, 128, 64), (300, 64, 128)])
@pytest.mark.parametrize("forced", [0, 2])
def test_nothing_is_written_outside_the_outputs(L, d, block, forced):
    print(f"case L={L} d={d} block={block} forced kernel {forced}", flush=True)
    B, H = 1, 2
    binding.asa_test_force_fwd_kernel(forced)
    try:
        q, k, v, g = (util.dev_bf16(synth.make_iid((B, H, L, d), L + d, s)) for s in range(4))
        so, o, st_o = _guarded(B, H, L, d)
        slo, o_lo, _ = _guarded(B, H, L, d)
        sg, go, _ = _guarded(B, H, L, d)
        go.copy_(g)                                    # dO shares O's strides
        p = binding.Params(B=B, H=H, L=L, d=d, block=block, o_stride=st_o)
        mask = synth.random_block_mask(p.Nb, 0.6, seed=L, slabs=B * H)
        bufs = util.lists_from_mask(p, mask)
        lse_store = torch.full((B * H * L + 64,), float("nan"), dtype=torch.float32, device="cuda")
        lse = lse_store[32:32 + B * H * L].view(B * H, L)
        ws = binding.alloc_workspace(binding.asa_fwd_workspace_bytes(p))
        binding.asa_attn_fwd(p, q, k, v, bufs["row_ptr"], bufs["col_idx"], o, lse, ws, o_lo=o_lo)
        torch.cuda.synchronize()
        _canaries_intact(so, o, "O")
        _canaries_intact(slo, o_lo, "o_lo")
        assert torch.isnan(lse_store[:32]).all() and torch.isnan(lse_store[32 + B * H * L:]).all()
        assert torch.isfinite(lse).all()
        # backward: dQ, dK, dV through their own guarded buffers
        sq, dq, st_q = _guarded(B, H, L, d)
        sk, dk, _ = _guarded(B, H, L, d)
        sv, dv, _ = _guarded(B, H, L, d)
        qg, kg, vg = (_guarded(B, H, L, d) for _ in range(3))
        for (_, view, _), src in zip((qg, kg, vg), (q, k, v)):
            view.copy_(src)
        pb = binding.Params(B=B, H=H, L=L, d=d, block=block, q_stride=st_q, k_stride=st_q,
                            v_stride=st_q, o_stride=st_o)
        wsb = binding.alloc_workspace(binding.asa_bwd_workspace_bytes(pb))
        for lo in (o_lo, None):
            binding.asa_attn_bwd(pb, qg[1], kg[1], vg[1], o, go, lse, bufs["row_ptr"], bufs["col_idx"],
                                 bufs["col_ptr"], bufs["row_idx"], dq, dk, dv, wsb, o_lo=lo)
            torch.cuda.synchronize()
            for s_, t_, n_ in ((sq, dq, "dQ"), (sk, dk, "dK"), (sv, dv, "dV")):
                _canaries_intact(s_, t_, n_)
                assert torch.isfinite(t_.float()).all()
    finally:
        binding.asa_test_force_fwd_kernel(0)


def _valid_lists(p, bufs):
    S, Nb = p.B * p.H, p.Nb
    mask = bufs["mask"].cpu().numpy().reshape(S, Nb, Nb)
    rp = bufs["row_ptr"].cpu().numpy().reshape(S, Nb + 1)
    ci = bufs["col_idx"].cpu().numpy().reshape(S, Nb * Nb)
    cp = bufs["col_ptr"].cpu().numpy().reshape(S, Nb + 1)
    ri = bufs["row_idx"].cpu().numpy().reshape(S, Nb * Nb)
    assert set(np.unique(mask)) <= {0, 1}
    for s in range(S):
        assert rp[s, 0] == 0 and cp[s, 0] == 0
        assert (np.diff(rp[s]) >= 1).all(), "a query block without a key block"
        assert rp[s, -1] == cp[s, -1] == mask[s].sum()
        for i in range(Nb):
            cols = ci[s, rp[s, i]:rp[s, i + 1]]
            assert (np.diff(cols) > 0).all() and cols.min() >= 0 and cols.max() < Nb
            assert np.array_equal(np.nonzero(mask[s, i])[0], cols)
            rows = ri[s, cp[s, i]:cp[s, i + 1]]
            assert np.array_equal(np.nonzero(mask[s, :, i])[0], rows)


@pytest.mark.parametrize("L,d,block", [(1000, 128, 128), (700, 64, 64)])
def test_non_finite_q_and_k_still_give_a_valid_mask(L, d, block):
    """NaN and +-Inf in sampled and unsampled rows of Q and K: asa_build_mask finishes, every row
    keeps at least one block, and the mask, CSR and CSC describe the same set."""
    B, H = 1, 3
    qb, kb = (synth.make_iid((B, H, L, d), L, s) for s in range(2))
    qf, kf = synth.bf16_bits_to_f32(qb).copy(), synth.bf16_bits_to_f32(kb).copy()
    stride = block // 16
    qf[0, 0, 0, 3] = np.nan                      # a sampled query row (offset 0 of block 0)
    qf[0, 0, stride * 5 + 1, 0] = np.inf         # an unsampled row
    kf[0, 0, block + stride * 2, 7] = np.nan     # a sampled key of block 1
    kf[0, 1, 2 * block, :] = np.inf              # a whole sampled key row
    kf[0, 1, 3 * block, 1] = -np.inf
    qf[0, 2, :, :] = np.nan                      # a head that is all NaN
    q, k = (util.dev_bf16(synth.f32_to_bf16_bits(x)) for x in (qf, kf))
    for r_min, r_max, tau in ((0.0, 1.0, 0.9), (0.25, 0.25, 0.9), (0.0, 0.5, 2.0)):
        p = binding.Params(B=B, H=H, L=L, d=d, block=block, tau=tau, r_min=r_min, r_max=r_max)
        bufs = binding.alloc_index_lists(p)
        ws = binding.alloc_workspace(binding.asa_mask_workspace_bytes(p))
        binding.asa_build_mask(p, q, k, bufs["mask"], bufs["row_ptr"], bufs["col_idx"], bufs["col_ptr"],
                               bufs["row_idx"], None, ws)
        torch.cuda.synchronize()
        _valid_lists(p, bufs)
