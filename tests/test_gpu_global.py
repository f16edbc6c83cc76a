"""GPU parity: ASA with global tokens (ASA_G, Sec. 3.3) vs the numpy oracle."""

import numpy as np
import pytest
import torch

from oracle import global_tokens as og
from paper_2508_10774_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu


def _pooled(p, n, k, v):
    G = binding.asa_global_token_count(p, n)
    kg = torch.full((p.B, p.H, G, p.d), float("nan"), dtype=torch.bfloat16, device="cuda")
    vg = torch.full_like(kg, float("nan"))
    binding.asa_global_tokens(p, n, k, v, kg, vg)
    torch.cuda.synchronize()
    return kg, vg


def _run_fwd_g(p, n, q, k, v, bufs, with_lo=False):
    kg, vg = _pooled(p, n, k, v)
    o = torch.full((p.B, p.H, p.L, p.d), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((p.B * p.H, p.L), float("nan"), dtype=torch.float32, device="cuda")
    o_lo = torch.empty_like(o) if with_lo else None
    ws = binding.alloc_workspace(binding.asa_fwd_g_workspace_bytes(p, n))
    binding.asa_attn_fwd_g(p, n, q, k, v, kg, vg, bufs["row_ptr"], bufs["col_idx"], o, lse, ws, o_lo=o_lo)
    torch.cuda.synchronize()
    return o, lse, o_lo, kg, vg


@pytest.mark.parametrize("L,d,block,n", [(1000, 128, 128, 128), (520, 64, 64, 16), (333, 128, 64, 50)])
def test_pooled_tokens_are_the_rounded_window_means(L, d, block, n):
    print(f"case pool L={L} d={d} block={block} n={n}", flush=True)
    p = binding.Params(B=1, H=2, L=L, d=d, block=block)
    kb, vb = (synth.make_iid((1, 2, L, d), 21, s) for s in range(2))
    kg, vg = _pooled(p, n, util.dev_bf16(kb), util.dev_bf16(vb))
    Lg = og.n_windows(L, n)
    assert kg.shape[2] == -(-Lg // block) * block
    for got, src in ((kg, kb), (vg, vb)):
        g = util.host_f32(got)
        assert (g[:, :, Lg:] == 0).all()                      # padding rows are zero
        for h in range(2):
            want, cnt = og.pool(synth.bf16_bits_to_f32(src[0, h]), n)
            assert cnt[-1] == L - (Lg - 1) * n
            diff = np.abs(g[0, h, :Lg] - want)
            # the GPU sums in fp32, the oracle in fp64: a mean that lands within 2^-24 of a bf16
            # rounding boundary may go the other way (one bf16 step), and only rarely
            assert (diff <= np.abs(want) * 2.0 ** -7 + 1e-30).all()
            assert (diff > 0).mean() < 2e-3


@pytest.mark.parametrize("B,H,L,d,block,n,dens", [
    (1, 2, 1024, 64, 64, 64, 0.4),       # window = block, exact multiples
    (1, 2, 1000, 128, 128, 128, 0.5),    # ragged last block and last window (104 tokens)
    (2, 1, 300, 64, 128, 16, 0.6),       # 19 pooled tokens in one padded pooled block
    (1, 2, 520, 128, 64, 8, 0.5),        # 65 pooled tokens: two pooled blocks, the second almost empty
    (1, 1, 200, 128, 128, 1, 1.0),       # n = 1: every token is its own pooled token
])
def test_fwd_global_tokens(B, H, L, d, block, n, dens):
    print(f"case B={B} H={H} L={L} d={d} block={block} n={n} dens={dens}", flush=True)
    p = binding.Params(B=B, H=H, L=L, d=d, block=block)
    qb, kb, vb = (synth.make_iid((B, H, L, d), L + d + n, s) for s in range(3))
    mask = synth.random_block_mask(p.Nb, dens, seed=L, slabs=B * H)
    mask[0, 0, :] = 0                     # a query block that sees the pooled tokens only
    bufs = util.lists_from_mask(p, mask, with_csc=False)
    o, lse, _, _, _ = _run_fwd_g(p, n, *(util.dev_bf16(x) for x in (qb, kb, vb)), bufs)
    qf, kf, vf = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb))
    m3 = mask.reshape(-1, p.Nb, p.Nb)
    for b in range(B):
        for h in range(H):
            want_o, want_lse = og.attn_fwd_g(qf[b, h], kf[b, h], vf[b, h], m3[b * H + h], block, n)
            e = util.assert_close_bf16(util.host_f32(o)[b, h], want_o, f"O[{b},{h}]")
            dl = np.abs(lse[b * H + h].cpu().numpy() - want_lse).max()
            print(f"  slab {b},{h}: O max-abs {e[0]:.2e}, LSE {dl:.2e}", flush=True)
            assert dl <= util.LSE_ABS


def test_fwd_global_tokens_dense_lists_and_residual():
    p = binding.Params(B=1, H=1, L=640, d=128, block=128)
    n = 32
    qb, kb, vb = (synth.make_iid((1, 1, 640, 128), 77, s) for s in range(3))
    q, k, v = (util.dev_bf16(x) for x in (qb, kb, vb))
    full = util.lists_from_mask(p, np.ones((1, 5, 5), np.uint8), with_csc=False)
    o_ref, lse_ref, lo_ref, _, _ = _run_fwd_g(p, n, q, k, v, full, with_lo=True)
    o, lse, lo, _, _ = _run_fwd_g(p, n, q, k, v, {"row_ptr": None, "col_idx": None}, with_lo=True)
    assert torch.equal(o.view(torch.int16), o_ref.view(torch.int16))
    assert torch.equal(lo.view(torch.int16), lo_ref.view(torch.int16))
    assert torch.equal(lse, lse_ref)
    qf, kf, vf = (synth.bf16_bits_to_f32(x)[0, 0] for x in (qb, kb, vb))
    want_o, _ = og.attn_fwd_g(qf, kf, vf, np.ones((5, 5), np.uint8), 128, n)
    # o + o_lo carries about 16 significant bits of the fp32 result
    both = util.host_f32(o)[0, 0].astype(np.float64) + util.host_f32(lo)[0, 0]
    assert np.abs(both - want_o).max() < 2e-3


def _run_bwd_g(p, n, q, k, v, g, bufs, with_lo=True):
    o, lse, o_lo, kg, vg = _run_fwd_g(p, n, q, k, v, bufs, with_lo=True)
    if not with_lo:
        o_lo = None          # the backward then forms Delta from the tiles (pooled ones included)
    dq = torch.full_like(q, float("nan"))
    dk = torch.full_like(k, float("nan"))
    dv = torch.full_like(v, float("nan"))
    ws = binding.alloc_workspace(binding.asa_bwd_g_workspace_bytes(p, n))
    binding.asa_attn_bwd_g(p, n, q, k, v, kg, vg, o, g, lse, bufs["row_ptr"], bufs["col_idx"],
                           bufs["col_ptr"], bufs["row_idx"], dq, dk, dv, ws, o_lo=o_lo)
    torch.cuda.synchronize()
    return [util.host_f32(x) for x in (dq, dk, dv)]


@pytest.mark.parametrize("B,H,L,d,block,n,dens", [
    (1, 2, 1024, 64, 64, 64, 0.4),
    (1, 2, 1000, 128, 128, 128, 0.5),    # ragged last block and last window
    (2, 1, 300, 64, 128, 16, 0.6),
    (1, 1, 520, 128, 64, 8, 0.5),        # two pooled blocks
])
def test_bwd_global_tokens(B, H, L, d, block, n, dens):
    print(f"case B={B} H={H} L={L} d={d} block={block} n={n} dens={dens}", flush=True)
    p = binding.Params(B=B, H=H, L=L, d=d, block=block)
    qb, kb, vb, gb = (synth.make_iid((B, H, L, d), L + d + n, s) for s in range(4))
    mask = synth.random_block_mask(p.Nb, dens, seed=L, slabs=B * H)
    mask[0, 0, :] = 0                     # a query block that sees the pooled tokens only
    mask[0, :, -1] = 0                    # a key block that gets gradient through the pooling only
    bufs = util.lists_from_mask(p, mask)
    dev = [util.dev_bf16(x) for x in (qb, kb, vb, gb)]
    qf, kf, vf, gf = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb, gb))
    m3 = mask.reshape(-1, p.Nb, p.Nb)
    want = {(b, h): og.attn_bwd_g(qf[b, h], kf[b, h], vf[b, h], gf[b, h], m3[b * H + h], block, n)
            for b in range(B) for h in range(H)}
    for with_lo in (True, False):
        dq, dk, dv = _run_bwd_g(p, n, *dev, bufs, with_lo=with_lo)
        for (b, h), (wq, wk, wv) in want.items():
            tag = f"[{b},{h}]" + ("" if with_lo else " (no o_lo)")
            util.assert_close_bf16(dq[b, h], wq, "dQ" + tag)
            util.assert_close_bf16(dk[b, h], wk, "dK" + tag)
            util.assert_close_bf16(dv[b, h], wv, "dV" + tag)


def test_bwd_global_tokens_dense_lists():
    p = binding.Params(B=1, H=1, L=384, d=64, block=64)
    n = 32
    qb, kb, vb, gb = (synth.make_iid((1, 1, 384, 64), 5, s) for s in range(4))
    t = [util.dev_bf16(x) for x in (qb, kb, vb, gb)]
    full = util.lists_from_mask(p, np.ones((1, 6, 6), np.uint8))
    none = {"row_ptr": None, "col_idx": None, "col_ptr": None, "row_idx": None}
    want = _run_bwd_g(p, n, *t, full)
    got = _run_bwd_g(p, n, *t, none)
    for a, b, name in zip(got, want, ("dQ", "dK", "dV")):
        assert np.array_equal(a, b), name
