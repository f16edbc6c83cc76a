"""asa_reorder_tokens and the Gilbert order on the GPU: the gather is exact (rows are copied), and
the rearranged tokens go through mask, forward and back like any others."""

import numpy as np
import pytest
import torch

import oracle
from oracle import gilbert
from paper_2508_10774_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,H,grid,n_prefix,d", [
    (1, 2, (4, 16, 16), 0, 64), (2, 3, (3, 5, 7), 11, 128), (1, 1, (1, 1, 1), 0, 64),
    (1, 2, (5, 9, 13), 0, 128)])
def test_reorder_matches_the_oracle_bit_for_bit(B, H, grid, n_prefix, d):
    L = n_prefix + grid[0] * grid[1] * grid[2]
    p = binding.Params(B=B, H=H, L=L, d=d, block=64)
    bits = [synth.make_iid((B, H, L, d), seed=3, stream=t) for t in range(3)]
    order, inverse = binding.asa_gilbert_order(*grid, n_prefix)
    want_order, _ = gilbert.token_order(grid, n_prefix)
    assert np.array_equal(order.numpy(), want_order)
    src = [util.dev_bf16(b) for b in bits]
    dst = [torch.full_like(t, float("nan")) for t in src]
    binding.asa_reorder_tokens(p, src, dst, order.cuda())
    back = [torch.full_like(t, float("nan")) for t in src]
    binding.asa_reorder_tokens(p, dst, back, inverse.cuda())
    torch.cuda.synchronize()
    for t in range(3):
        want = gilbert.permute_tokens(bits[t], want_order)
        got = dst[t].view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, want), t
        assert np.array_equal(back[t].view(torch.int16).cpu().numpy().view(np.uint16), bits[t]), t


def test_reorder_strided_source_and_bad_index_entries():
    B, H, L, d = 2, 2, 300, 64
    p = binding.Params(B=B, H=H, L=L, d=d, block=64)
    # source laid out [B, L, H, d] (as a projection writes it), destination packed [B, H, L, d]
    bits = synth.make_iid((B, L, H, d), seed=9)
    src = util.dev_bf16(bits)
    dst = torch.full((B, H, L, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    rng = np.random.default_rng(1)
    idx = rng.permutation(L).astype(np.int32)
    idx[5], idx[17] = -1, L       # outside [0, L): zero rows
    binding.asa_reorder_tokens(p, [src], [dst], torch.from_numpy(idx).cuda(),
                               src_stride=(L * H * d, d, H * d))
    torch.cuda.synchronize()
    got = dst.view(torch.int16).cpu().numpy().view(np.uint16)
    want = np.transpose(bits, (0, 2, 1, 3))[:, :, np.clip(idx, 0, L - 1), :].copy()
    want[:, :, 5, :] = 0
    want[:, :, 17, :] = 0
    assert np.array_equal(got, want)


def test_reorder_three_tensors_into_a_strided_destination():
    B, H, L, d = 1, 3, 777, 64
    p = binding.Params(B=B, H=H, L=L, d=d, block=64)
    bits = [synth.make_iid((B, H, L, d), seed=21, stream=t) for t in range(3)]
    src = [util.dev_bf16(b) for b in bits]
    # destination laid out [B, L, H, d]
    dst = [torch.full((B, L, H, d), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(3)]
    idx = np.random.default_rng(5).permutation(L).astype(np.int32)
    binding.asa_reorder_tokens(p, src, dst, torch.from_numpy(idx).cuda(), dst_stride=(L * H * d, d, H * d))
    torch.cuda.synchronize()
    for t in range(3):
        got = dst[t].permute(0, 2, 1, 3).contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, bits[t][:, :, idx, :]), t


def test_reorder_rejects_bad_arguments():
    p = binding.Params(B=1, H=1, L=64, d=64, block=64)
    x = torch.zeros((1, 1, 64, 64), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros_like(x)
    idx = torch.arange(64, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.AsaError):
        binding.asa_reorder_tokens(p, [x], [x], idx)                      # in place
    with pytest.raises(binding.AsaError):
        binding.asa_reorder_tokens(p, [x, x, x, x], [y, y, y, y], idx)    # more than three
    with pytest.raises(binding.AsaError):
        binding.asa_reorder_tokens(p, [x], [y], idx, src_stride=(4096, 4096, 60))


def test_rearranged_tokens_through_mask_and_forward():
    """Tiny workload: Gilbert order -> mask -> forward -> inverse order, against the oracle doing
    the same steps; and the density at equal tau drops as the paper's ablation says."""
    w = synth.TINY
    qb, kb, vb = synth.make_qkv(w, seed=2)
    p = binding.Params(B=w.B, H=w.H, L=w.L, d=w.d, block=w.block, k_samples=w.k_samples, tau=0.9)
    order, inverse = binding.asa_gilbert_order(*w.grid, w.n_text)
    q, k, v = (util.dev_bf16(x) for x in (qb, kb, vb))
    qg, kg, vg = (torch.empty_like(t) for t in (q, k, v))
    binding.asa_reorder_tokens(p, [q, k, v], [qg, kg, vg], order.cuda())
    bufs = binding.alloc_index_lists(p)
    ws = binding.alloc_workspace(binding.asa_mask_workspace_bytes(p))
    binding.asa_build_mask(p, qg, kg, bufs["mask"], bufs["row_ptr"], bufs["col_idx"], bufs["col_ptr"],
                           bufs["row_idx"], workspace=ws)
    o_g, lse = util.run_fwd(p, qg, kg, vg, bufs)
    o = torch.empty_like(o_g)
    binding.asa_reorder_tokens(p, [o_g], [o], inverse.cuda())
    torch.cuda.synchronize()

    o_order, o_inverse = gilbert.token_order(w.grid, w.n_text)
    qf, kf, vf = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb))
    qo, ko, vo = (gilbert.permute_tokens(x, o_order) for x in (qf, kf, vf))
    offs = synth.default_sample_offsets(w.block, w.k_samples)
    mask_o, P = oracle.build_mask(qo, ko, w.block, offs, 0.9)
    mask_g = bufs["mask"].cpu().numpy().reshape(mask_o.shape)
    exact, excused, failed = util.classify_mask_rows(P, mask_o, mask_g, 0.9)
    assert not failed, failed
    # forward on the library's own mask, compared with the oracle on that same mask
    want = np.empty((w.B, w.H, w.L, w.d), dtype=np.float64)
    for b in range(w.B):
        for h in range(w.H):
            out = oracle.attn_fwd(qo[b, h], ko[b, h], vo[b, h], mask_g[b, h], w.block)
            want[b, h] = out[0]
    want = gilbert.permute_tokens(want, o_inverse)
    util.assert_close_bf16(util.host_f32(o), want, "O in raster order")
    mask_raster, _ = oracle.build_mask(qf, kf, w.block, offs, 0.9)
    assert mask_g.mean() < mask_raster.mean()


def test_mfma_rate_probe_runs_and_checks_its_arguments():
    sink = torch.zeros(4 * 512, dtype=torch.float32, device="cuda")
    flop = binding.asa_mfma_rate_probe(4, 8, sink)
    torch.cuda.synchronize()
    assert flop == 4 * 8 * 4 * 8 * 2 * 32 * 32 * 16
    assert torch.isfinite(sink).all()
    # with idle pauses or a vector stream beside it, four wavefronts per workgroup count
    for kw in ({"idle_sleep": 3}, {"vector_stream": True}, {"idle_sleep": 7, "vector_stream": True}):
        flop = binding.asa_mfma_rate_probe(4, 8, sink, **kw)
        torch.cuda.synchronize()
        assert flop == 4 * 4 * 4 * 8 * 2 * 32 * 32 * 16
        assert torch.isfinite(sink).all()
    with pytest.raises(binding.AsaError):
        binding.asa_mfma_rate_probe(4, 8, sink, idle_sleep=8)
    with pytest.raises(binding.AsaError):
        binding.asa_mfma_rate_probe(0, 8, sink)
    with pytest.raises(binding.AsaError):
        binding.asa_mfma_rate_probe(4, 0, sink)
