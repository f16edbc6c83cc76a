"""GPU parity: block-sparse attention backward (dQ, dK, dV) vs the CPU oracle."""

import numpy as np
import pytest
import torch

import oracle
from paper_2508_10774_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu


def _run(p, qb, kb, vb, gb, mask, with_lo=True):
    bufs = util.lists_from_mask(p, mask)
    q, k, v, g = (util.dev_bf16(x) for x in (qb, kb, vb, gb))
    if with_lo:
        o, lse, o_lo = util.run_fwd(p, q, k, v, bufs, with_lo=True)
    else:
        (o, lse), o_lo = util.run_fwd(p, q, k, v, bufs), None
    dq, dk, dv = util.run_bwd(p, q, k, v, o, lse, g, bufs, o_lo=o_lo)
    return [util.host_f32(x) for x in (dq, dk, dv)]


def _check_bwd(p, qb, kb, vb, gb, mask, with_lo=True, use_mag=False):
    """use_mag: the element-wise allowance of util.assert_close_bf16 (inputs with large keys and
    gradients); otherwise the plain 2e-2 / 2e-3 on every element."""
    dq, dk, dv = _run(p, qb, kb, vb, gb, mask, with_lo)
    qf, kf, vf, gf = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb, gb))
    m3 = mask.reshape(-1, p.Nb, p.Nb)
    for b in range(p.B):
        for h in range(p.H):
            wq, wk, wv, mq, mk, mv = oracle.attn_bwd(qf[b, h], kf[b, h], vf[b, h], gf[b, h],
                                                     m3[b * p.H + h], p.block,
                                                     p.scale if p.scale else None, with_mag=True)
            tag = f"[{b},{h}]" + ("" if with_lo else " (no o_lo)")
            util.assert_close_bf16(dq[b, h], wq, "dQ" + tag, mq if use_mag else None)
            util.assert_close_bf16(dk[b, h], wk, "dK" + tag, mk if use_mag else None)
            util.assert_close_bf16(dv[b, h], wv, "dV" + tag, mv if use_mag else None)


@pytest.mark.parametrize("B,H,L,d,block,dens", [
    (1, 2, 1024, 64, 64, 0.4),
    (1, 2, 1000, 128, 128, 0.5),     # ragged tail
    (2, 1, 300, 64, 128, 0.6),
    (1, 2, 520, 128, 64, 0.5),
    (1, 1, 64, 64, 64, 1.0),
    (1, 1, 3, 128, 128, 1.0),
])
def test_bwd_random_masks(B, H, L, d, block, dens):
    print(f"case B={B} H={H} L={L} d={d} block={block} dens={dens}", flush=True)
    p = binding.Params(B=B, H=H, L=L, d=d, block=block)
    shape = (B, H, L, d)
    qb, kb, vb, gb = (synth.make_iid(shape, L + d, s) for s in range(4))
    mask = synth.random_block_mask(p.Nb, dens, seed=L, slabs=B * H)
    _check_bwd(p, qb, kb, vb, gb, mask)
    # without the saved low part of O the backward forms Delta from the tiles themselves
    _check_bwd(p, qb, kb, vb, gb, mask, with_lo=False)


@pytest.mark.parametrize("L,d,block", [(640, 128, 128), (333, 64, 64)])
def test_bwd_dense_specialisation_needs_no_lists(L, d, block):
    """All four list pointers NULL: the same tiles in the same order as a full mask's lists,
    hence bit-identical gradients (the full-mask path is checked against the oracle above)."""
    print(f"case dense L={L} d={d} block={block}", flush=True)
    p = binding.Params(B=1, H=2, L=L, d=d, block=block)
    shape = (1, 2, L, d)
    qb, kb, vb, gb = (synth.make_iid(shape, L + d, s) for s in range(4))
    q, k, v, g = (util.dev_bf16(x) for x in (qb, kb, vb, gb))
    mask = np.ones((2, p.Nb, p.Nb), np.uint8)
    full = util.lists_from_mask(p, mask)
    none = {"row_ptr": None, "col_idx": None, "col_ptr": None, "row_idx": None}
    o, lse, o_lo = util.run_fwd(p, q, k, v, none, with_lo=True)
    want = util.run_bwd(p, q, k, v, o, lse, g, full, o_lo=o_lo)
    got = util.run_bwd(p, q, k, v, o, lse, g, none, o_lo=o_lo)
    for a, b, name in zip(got, want, ("dQ", "dK", "dV")):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)), name
    qf, kf, vf, gf = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb, gb))
    wq, wk, wv = oracle.attn_bwd(qf[0, 1], kf[0, 1], vf[0, 1], gf[0, 1], mask[1], block, None)
    util.assert_close_bf16(util.host_f32(got[0])[0, 1], wq, "dense dQ")
    util.assert_close_bf16(util.host_f32(got[1])[0, 1], wk, "dense dK")
    util.assert_close_bf16(util.host_f32(got[2])[0, 1], wv, "dense dV")


def test_bwd_empty_rows_and_columns():
    p = binding.Params(B=1, H=1, L=384, d=64, block=64)
    shape = (1, 1, 384, 64)
    qb, kb, vb, gb = (synth.make_iid(shape, 77, s) for s in range(4))
    mask = synth.random_block_mask(6, 0.5, seed=7, slabs=1)
    mask[0, 2, :] = 0        # query block 2 sees nothing: dQ rows are zero
    mask[0, :, 4] = 0        # key block 4 is seen by nobody: dK, dV rows are zero
    mask[0, 0, 0] = mask[0, 1, 1] = mask[0, 3, 3] = mask[0, 4, 5] = mask[0, 5, 5] = 1
    dq, dk, dv = _run(p, qb, kb, vb, gb, mask)
    assert (dq[0, 0, 128:192] == 0).all()
    assert (dk[0, 0, 256:320] == 0).all() and (dv[0, 0, 256:320] == 0).all()
    _check_bwd(p, qb, kb, vb, gb, mask)


def test_bwd_tiny_workload_with_oracle_mask():
    w = synth.TINY
    qb, kb, vb = synth.make_qkv(w, seed=0)
    gb = synth.make_do(w, seed=0)
    p = binding.Params(B=w.B, H=w.H, L=w.L, d=w.d, block=w.block)
    mask, _ = oracle.build_mask(synth.bf16_bits_to_f32(qb), synth.bf16_bits_to_f32(kb), w.block,
                                synth.default_sample_offsets(w.block, w.k_samples), tau=0.9)
    _check_bwd(p, qb, kb, vb, gb, mask, use_mag=True)
    _check_bwd(p, qb, kb, vb, gb, mask, with_lo=False, use_mag=True)   # the plain call: no o_lo


def test_bwd_custom_scale_and_determinism():
    p = binding.Params(B=1, H=2, L=768, d=128, block=128, scale=0.05)
    shape = (1, 2, 768, 128)
    qb, kb, vb, gb = (synth.make_iid(shape, 9, s) for s in range(4))
    mask = synth.random_block_mask(p.Nb, 0.6, seed=9, slabs=2)
    _check_bwd(p, qb, kb, vb, gb, mask)
    a = _run(p, qb, kb, vb, gb, mask)
    b = _run(p, qb, kb, vb, gb, mask)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("L,d,block", [(700, 128, 128), (333, 64, 64), (450, 128, 64)])
def test_bwd_packed_qkv_layout_with_different_strides_per_tensor(L, d, block):
    """Q, K, V live interleaved in one [B, L, 3, H, d] buffer (so do dQ, dK, dV), O and dO in a
    [B, L, H, d] buffer: the row pitch of Q / K / V (3 H d) differs from that of O / dO (H d),
    the tail block is ragged, and every gradient is written through its own strides."""
    print(f"case packed L={L} d={d} block={block}", flush=True)
    B, H = 1, 2
    shape = (B, H, L, d)
    qb, kb, vb, gb = (synth.make_iid(shape, L + d, 40 + s) for s in range(4))
    st_qkv = (L * 3 * H * d, d, 3 * H * d)
    st_o = (L * H * d, d, H * d)
    p = binding.Params(B=B, H=H, L=L, d=d, block=block, q_stride=st_qkv, k_stride=st_qkv,
                       v_stride=st_qkv, o_stride=st_o)
    mask = synth.random_block_mask(p.Nb, 0.5, seed=L, slabs=B * H)
    bufs = util.lists_from_mask(p, mask)
    qkv = torch.empty((B, L, 3, H, d), dtype=torch.bfloat16, device="cuda")
    for i, x in enumerate((qb, kb, vb)):
        qkv[:, :, i] = util.dev_bf16(x).permute(0, 2, 1, 3)
    q, k, v = (qkv[:, :, i].permute(0, 2, 1, 3) for i in range(3))          # views [B, H, L, d]
    g = util.dev_bf16(gb).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    o = torch.zeros((B, L, H, d), dtype=torch.bfloat16, device="cuda").permute(0, 2, 1, 3)
    o_lo = torch.zeros((B, L, H, d), dtype=torch.bfloat16, device="cuda").permute(0, 2, 1, 3)
    lse = torch.empty((B * H, L), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(binding.asa_fwd_workspace_bytes(p))
    binding.asa_attn_fwd(p, q, k, v, bufs["row_ptr"], bufs["col_idx"], o, lse, ws, o_lo=o_lo)
    dqkv = torch.full((B, L, 3, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    dq, dk, dv = (dqkv[:, :, i].permute(0, 2, 1, 3) for i in range(3))
    ws = binding.alloc_workspace(binding.asa_bwd_workspace_bytes(p))
    binding.asa_attn_bwd(p, q, k, v, o, g, lse, bufs["row_ptr"], bufs["col_idx"], bufs["col_ptr"],
                         bufs["row_idx"], dq, dk, dv, ws, o_lo=o_lo)
    torch.cuda.synchronize()
    got = [util.host_f32(x.contiguous()) for x in (dq, dk, dv)]
    qf, kf, vf, gf = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb, gb))
    for h in range(H):
        want = oracle.attn_bwd(qf[0, h], kf[0, h], vf[0, h], gf[0, h], mask[h], block, None)
        for name, a, w in zip(("dQ", "dK", "dV"), got, want):
            util.assert_close_bf16(a[0, h], w, f"packed {name}[{h}]")
