"""GPU parity: block-sparse attention forward vs the CPU oracle, through the C ABI."""

import numpy as np
import pytest
import torch

import oracle
from paper_2508_10774_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["auto", "pingpong"])
def kernel_choice(request):
    """Every test of this module runs twice: with the library's own choice of forward kernel (short
    lists go to the lock-step kernel) and with the ping-pong kernel forced, so that both kernels
    see every edge case."""
    binding.asa_test_force_fwd_kernel(2 if request.param == "pingpong" else 0)
    yield request.param
    binding.asa_test_force_fwd_kernel(0)


def _case(B, H, L, d, block, seed):
    shape = (B, H, L, d)
    q, k, v = (synth.make_iid(shape, seed, s) for s in range(3))
    return q, k, v


def _check_fwd(p, qb, kb, vb, mask, heads=None, qblocks=None):
    bufs = util.lists_from_mask(p, mask, with_csc=False)
    o, lse = util.run_fwd(p, util.dev_bf16(qb), util.dev_bf16(kb), util.dev_bf16(vb), bufs)
    o = util.host_f32(o)
    lse = lse.cpu().numpy()
    qf, kf, vf = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb))
    scale = p.scale if p.scale else None
    worst = (0.0, 0.0)
    for b in range(p.B):
        for h in (heads if heads is not None else range(p.H)):
            s = b * p.H + h
            want, wl = oracle.attn_fwd(qf[b, h], kf[b, h], vf[b, h], mask.reshape(-1, p.Nb, p.Nb)[s],
                                       p.block, scale, qblocks)
            rows = ~np.isnan(wl)
            e = util.assert_close_bf16(o[b, h][rows], want[rows], f"O[{b},{h}]")
            worst = max(worst, e)
            fin = np.isfinite(wl[rows])
            assert np.abs(lse[s][rows][fin] - wl[rows][fin]).max() <= util.LSE_ABS
            assert np.array_equal(np.isneginf(lse[s][rows]), np.isneginf(wl[rows]))
    return worst


@pytest.mark.parametrize("B,H,L,d,block,dens", [
    (1, 2, 1024, 64, 64, 0.4),      # several tiles, exact multiple
    (1, 2, 1000, 128, 128, 0.5),    # ragged tail: last block 104 valid
    (2, 2, 300, 64, 128, 0.6),      # block 128 with d 64, tail 44
    (1, 3, 520, 128, 64, 0.5),      # block 64 with d 128, tail 8
    (1, 1, 64, 64, 64, 1.0),        # a single block
    (1, 1, 1, 128, 128, 1.0),       # a single token
])
def test_fwd_random_masks(B, H, L, d, block, dens):
    print(f"case B={B} H={H} L={L} d={d} block={block} dens={dens}", flush=True)
    p = binding.Params(B=B, H=H, L=L, d=d, block=block)
    qb, kb, vb = _case(B, H, L, d, block, seed=L + d)
    mask = synth.random_block_mask(p.Nb, dens, seed=L, slabs=B * H)
    _check_fwd(p, qb, kb, vb, mask)


def test_fwd_all_blocks_kept_is_dense_attention():
    p = binding.Params(B=1, H=2, L=640, d=128, block=128)
    qb, kb, vb = _case(1, 2, 640, 128, 128, seed=3)
    mask = np.ones((2, p.Nb, p.Nb), np.uint8)
    bufs = util.lists_from_mask(p, mask, with_csc=False)
    o, _ = util.run_fwd(p, util.dev_bf16(qb), util.dev_bf16(kb), util.dev_bf16(vb), bufs)
    qf, kf, vf = (torch.from_numpy(synth.bf16_bits_to_f32(x).astype(np.float64)) for x in (qb, kb, vb))
    want = torch.nn.functional.scaled_dot_product_attention(qf, kf, vf).numpy()
    util.assert_close_bf16(util.host_f32(o), want, "dense O")


@pytest.mark.parametrize("L,d,block", [(640, 128, 128), (1000, 64, 64), (333, 128, 64)])
def test_fwd_dense_specialisation_needs_no_lists(L, d, block):
    """row_ptr = col_idx = NULL: every key block.  Same tiles in the same order as a full mask's
    lists, so bit-identical to that call; and equal to plain soft-max attention."""
    print(f"case dense L={L} d={d} block={block}", flush=True)
    p = binding.Params(B=1, H=2, L=L, d=d, block=block)
    qb, kb, vb = _case(1, 2, L, d, block, seed=11)
    q, k, v = (util.dev_bf16(x) for x in (qb, kb, vb))
    full = util.lists_from_mask(p, np.ones((2, p.Nb, p.Nb), np.uint8), with_csc=False)
    o_ref, lse_ref = util.run_fwd(p, q, k, v, full)
    o, lse = util.run_fwd(p, q, k, v, {"row_ptr": None, "col_idx": None})
    assert torch.equal(o.view(torch.int16), o_ref.view(torch.int16))
    assert torch.equal(lse, lse_ref)
    qf, kf, vf = (torch.from_numpy(synth.bf16_bits_to_f32(x).astype(np.float64)) for x in (qb, kb, vb))
    want = torch.nn.functional.scaled_dot_product_attention(qf, kf, vf).numpy()
    util.assert_close_bf16(util.host_f32(o), want, "dense O")


def test_fwd_single_stage_kernel_is_still_correct():
    """The kernel that takes over for slabs of 4 GiB and more, forced by its switch."""
    binding.asa_test_force_fwd_kernel(1)
    p = binding.Params(B=1, H=2, L=1000, d=128, block=128)
    qb, kb, vb = _case(1, 2, 1000, 128, 128, seed=5)
    mask = synth.random_block_mask(p.Nb, 0.5, seed=5, slabs=2)
    _check_fwd(p, qb, kb, vb, mask)
    p = binding.Params(B=1, H=1, L=520, d=64, block=64)
    qb, kb, vb = _case(1, 1, 520, 64, 64, seed=6)
    _check_fwd(p, qb, kb, vb, synth.random_block_mask(p.Nb, 0.6, seed=6, slabs=1))


@pytest.mark.parametrize("L,d,block", [(1024, 64, 64), (520, 128, 64), (300, 64, 128)])
def test_fwd_ping_pong_kernel_at_the_sizes_where_it_is_not_the_default(L, d, block):
    binding.asa_test_force_fwd_kernel(2)
    p = binding.Params(B=1, H=2, L=L, d=d, block=block)
    qb, kb, vb = _case(1, 2, L, d, block, seed=L)
    _check_fwd(p, qb, kb, vb, synth.random_block_mask(p.Nb, 0.5, seed=L, slabs=2))


def test_fwd_each_slab_goes_to_the_kernel_that_suits_its_lists(kernel_choice):
    """Block 128 / d 128 without a lower retention clamp: both kernels are launched and each takes
    the (batch, head) slabs whose rows are long / short for it.  Head 0 keeps 32 of 40 blocks per
    row (ping-pong kernel), head 1 keeps 6 (lock-step kernel), head 2 sits just below the
    switch-over (17 per row), head 3 just above (18); every row must come from exactly one."""
    if kernel_choice != "auto":
        pytest.skip("the choice is what is tested")
    L, H = 128 * 40 - 9, 4
    p = binding.Params(B=1, H=H, L=L, d=128, block=128)
    qb, kb, vb = _case(1, H, L, 128, 128, seed=77)
    mask = np.zeros((H, p.Nb, p.Nb), np.uint8)
    rng = np.random.default_rng(7)
    for h, m in enumerate((32, 6, 17, 18)):
        for i in range(p.Nb):
            mask[h, i, rng.choice(p.Nb, size=m, replace=False)] = 1
    _check_fwd(p, qb, kb, vb, mask)


def test_fwd_tiny_workload_with_oracle_mask():
    w = synth.TINY
    qb, kb, vb = synth.make_qkv(w, seed=0)
    p = binding.Params(B=w.B, H=w.H, L=w.L, d=w.d, block=w.block)
    qf, kf = synth.bf16_bits_to_f32(qb), synth.bf16_bits_to_f32(kb)
    mask, _ = oracle.build_mask(qf, kf, w.block, synth.default_sample_offsets(w.block, w.k_samples),
                                tau=0.9)
    _check_fwd(p, qb, kb, vb, mask)


def test_fwd_peaked_logits_and_custom_scale():
    # large logits (shared smooth field) stress the running-maximum rescaling
    w = synth.Workload("t", 1, 2, 128, (2, 16, 16), 0, 128, 16)
    qb, kb, vb = synth.make_qkv(w, seed=5)
    p = binding.Params(B=1, H=2, L=w.L, d=128, block=128, scale=0.05)
    mask = synth.random_block_mask(p.Nb, 0.7, seed=9, slabs=2)
    _check_fwd(p, qb, kb, vb, mask)


def test_fwd_empty_row_gives_zero_and_minus_inf():
    p = binding.Params(B=1, H=1, L=256, d=64, block=64)
    qb, kb, vb = _case(1, 1, 256, 64, 64, seed=8)
    mask = synth.random_block_mask(4, 0.5, seed=1, slabs=1)
    mask[0, 2, :] = 0
    bufs = util.lists_from_mask(p, mask, with_csc=False)
    o, lse = util.run_fwd(p, util.dev_bf16(qb), util.dev_bf16(kb), util.dev_bf16(vb), bufs)
    assert (util.host_f32(o)[0, 0, 128:192] == 0).all()
    assert torch.isneginf(lse[0, 128:192]).all()
    _check_fwd(p, qb, kb, vb, mask)


def test_fwd_strided_inputs():
    # [B, L, H, d] storage viewed as [B, H, L, d]
    B, H, L, d, block = 1, 2, 384, 64, 64
    qb, kb, vb = _case(B, H, L, d, block, seed=12)
    st = (L * H * d, d, H * d)
    p = binding.Params(B=B, H=H, L=L, d=d, block=block, q_stride=st, k_stride=st, v_stride=st,
                       o_stride=st)
    mask = synth.random_block_mask(p.Nb, 0.5, seed=2, slabs=B * H)
    bufs = util.lists_from_mask(p, mask, with_csc=False)
    tq, tk, tv = (util.dev_bf16(x).permute(0, 2, 1, 3).contiguous() for x in (qb, kb, vb))
    o = torch.zeros((B, L, H, d), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B * H, L), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(binding.asa_fwd_workspace_bytes(p))
    binding.asa_attn_fwd(p, tq, tk, tv, bufs["row_ptr"], bufs["col_idx"], o, lse, ws)
    torch.cuda.synchronize()
    got = util.host_f32(o.permute(0, 2, 1, 3))
    qf, kf, vf = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb))
    for h in range(H):
        want, _ = oracle.attn_fwd(qf[0, h], kf[0, h], vf[0, h], mask[h], block)
        util.assert_close_bf16(got[0, h], want, f"strided O[{h}]")


def test_fwd_is_deterministic():
    p = binding.Params(B=1, H=2, L=1024, d=128, block=128)
    qb, kb, vb = _case(1, 2, 1024, 128, 128, seed=4)
    mask = synth.random_block_mask(p.Nb, 0.5, seed=4, slabs=2)
    bufs = util.lists_from_mask(p, mask, with_csc=False)
    args = [util.dev_bf16(x) for x in (qb, kb, vb)]
    o1, l1 = util.run_fwd(p, *args, bufs)
    o2, l2 = util.run_fwd(p, *args, bufs)
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)) and torch.equal(l1, l2)
