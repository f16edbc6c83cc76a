"""GPU parity: mask generation (importance map, threshold rule, index lists) vs the oracle."""

import numpy as np
import pytest
import torch

import oracle
from paper_2508_10774_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu

P_IMP_RTOL = 1e-4      # importance map: bf16 products summed in fp32 on the GPU, fp64 in the oracle


def _scores(rows, Nb, seed):
    rng = np.random.default_rng(seed)
    sc = (rng.random((rows, Nb), dtype=np.float32) ** 6).astype(np.float32)
    sc[::5] = np.round(sc[::5] * 16) / 16            # exact ties
    sc[1] = 0.0                                       # all-zero row
    sc[2] = np.float32(1.0 / 4096)                    # uniform row
    sc[3, ::3] = np.nan                               # NaN scores count as zero
    sc[4] = np.float32(1e-30) * rng.random(Nb, dtype=np.float32)   # tiny magnitudes
    sc[5, 0] = 1.0
    sc[5, 1:] *= 1e-9                                 # peaked row with a long small tail
    return sc


@pytest.mark.parametrize("Nb", [1, 16, 100, 256, 278, 1024])
@pytest.mark.parametrize("tau,r_min,r_max", [(0.9, 0, 1), (0.5, 0.1, 0.5), (0.999, 0, 0.25),
                                             (2.0, 0, 1), (0.0, 0, 1), (0.9, 0.25, 0.25)])
def test_rule_kernel_is_bit_exact(Nb, tau, r_min, r_max):
    print(f"case Nb={Nb} tau={tau} r=({r_min},{r_max})", flush=True)
    H = 3
    block = 64
    L = Nb * block - 5 if Nb > 1 else 40
    p = binding.Params(B=1, H=H, L=L, d=64, block=block, tau=tau, r_min=r_min, r_max=r_max)
    assert p.Nb == Nb
    sc = _scores(H * Nb, Nb, seed=Nb) if Nb >= 16 else np.random.default_rng(0).random(
        (H * Nb, Nb), dtype=np.float32)
    want, _ = oracle.mask_rule(sc, tau, r_min, r_max)
    got = torch.empty((H, Nb, Nb), dtype=torch.uint8, device="cuda")
    binding.asa_mask_from_scores(p, torch.from_numpy(sc).cuda(), got)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().reshape(-1, Nb), want)


@pytest.mark.parametrize("Nb", [2, 63, 64, 65, 127, 128, 129, 255, 257, 511, 512, 513, 1023])
def test_rule_kernel_at_the_edges_of_its_network_sizes(Nb):
    """The sorting network is built for 128, 256, 512 or 1024 keys; rows just below, at and just
    above those sizes (and rows shorter than a wavefront) against the oracle, bit for bit."""
    H, block = 2, 64
    p = binding.Params(B=1, H=H, L=Nb * block - 3, d=64, block=block, tau=0.8, r_min=0.05, r_max=0.9)
    assert p.Nb == Nb
    sc = _scores(H * Nb, Nb, seed=1000 + Nb) if Nb >= 16 else np.random.default_rng(Nb).random(
        (H * Nb, Nb), dtype=np.float32)
    want, _ = oracle.mask_rule(sc, 0.8, 0.05, 0.9)
    got = torch.empty((H, Nb, Nb), dtype=torch.uint8, device="cuda")
    binding.asa_mask_from_scores(p, torch.from_numpy(sc).cuda(), got)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().reshape(-1, Nb), want)


def test_rule_kernel_forced_prefix():
    Nb, block = 20, 64
    p = binding.Params(B=1, H=2, L=Nb * block, d=64, block=block, tau=0.6, n_prefix_dense=130)
    sc = _scores(2 * Nb, Nb, seed=3)
    want, _ = oracle.mask_rule(sc, 0.6)
    want = oracle.force_prefix(want.reshape(2, Nb, Nb), block, 130)
    got = torch.empty((2, Nb, Nb), dtype=torch.uint8, device="cuda")
    binding.asa_mask_from_scores(p, torch.from_numpy(sc).cuda(), got)
    assert np.array_equal(got.cpu().numpy(), want)
    assert want[:, :3, :].all() and want[:, :, :3].all()


@pytest.mark.parametrize("Nb,dens", [(1, 1.0), (16, 0.3), (257, 0.2), (1024, 0.05)])
def test_index_lists_match_the_mask(Nb, dens):
    print(f"case Nb={Nb}", flush=True)
    block = 64
    p = binding.Params(B=2, H=2, L=Nb * block, d=64, block=block)
    mask = synth.random_block_mask(Nb, dens, seed=Nb, slabs=4)
    if Nb > 4:
        mask[1, 3, :] = 0            # an empty row
        mask[2, :, 2] = 0            # an empty column
    bufs = util.lists_from_mask(p, mask)
    torch.cuda.synchronize()
    rp, ci = oracle.csr_from_mask(mask)
    cp, ri = oracle.csc_from_mask(mask)
    assert np.array_equal(bufs["row_ptr"].cpu().numpy(), rp)
    assert np.array_equal(bufs["col_ptr"].cpu().numpy(), cp)
    gci, gri = bufs["col_idx"].cpu().numpy(), bufs["row_idx"].cpu().numpy()
    for s in range(4):
        n = rp[s, -1]
        assert np.array_equal(gci[s, :n], ci[s, :n]) and np.array_equal(gri[s, :n], ri[s, :n])


def _build(p, qb, kb, want_csc=True):
    bufs = binding.alloc_index_lists(p, with_csc=want_csc)
    pimp = torch.empty((p.B * p.H, p.Nb, p.Nb), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(binding.asa_mask_workspace_bytes(p))
    binding.asa_build_mask(p, util.dev_bf16(qb), util.dev_bf16(kb), bufs["mask"], bufs["row_ptr"],
                           bufs["col_idx"], bufs.get("col_ptr"), bufs.get("row_idx"), pimp, ws)
    torch.cuda.synchronize()
    return bufs, pimp.cpu().numpy()


def _oracle_p(p, qb, kb, offs):
    qf, kf = synth.bf16_bits_to_f32(qb), synth.bf16_bits_to_f32(kb)
    out = np.empty((p.B * p.H, p.Nb, p.Nb), np.float32)
    for b in range(p.B):
        for h in range(p.H):
            out[b * p.H + h] = oracle.p_imp(qf[b, h], kf[b, h], p.block, offs,
                                            p.scale if p.scale else None)
    return out


def _check_build(p, qb, kb, offs, label):
    bufs, gp = _build(p, qb, kb)
    op = _oracle_p(p, qb, kb, offs)
    # (1) importance map
    nz = op > 1e-30
    rel = np.abs(gp[nz] - op[nz]) / op[nz]
    assert rel.max() <= P_IMP_RTOL, f"{label}: P_imp rel err {rel.max():.3e}"
    assert np.all(gp[~nz] <= 1e-29)
    # (2) the GPU mask is the oracle's rule applied to the GPU's own scores, bit for bit
    gm = bufs["mask"].cpu().numpy()
    self_rule, _ = oracle.mask_rule(gp, p.tau, p.r_min, p.r_max)
    assert np.array_equal(gm, self_rule), f"{label}: rule kernel differs on its own scores"
    # (3) against the oracle end to end: equal, or excused by sub-1e-6 score gaps
    om, _ = oracle.mask_rule(op, p.tau, p.r_min, p.r_max)
    exact, excused, failed = util.classify_mask_rows(op, om, gm, p.tau)
    print(f"{label}: mask rows exact={exact} excused={excused} failed={len(failed)} "
          f"P_imp max rel err={rel.max():.2e}", flush=True)
    assert not failed, f"{label}: rows {failed[:8]} differ beyond the score-gap allowance"
    # (4) index lists describe the GPU mask
    rp, ci = oracle.csr_from_mask(gm)
    cp, ri = oracle.csc_from_mask(gm)
    assert np.array_equal(bufs["row_ptr"].cpu().numpy(), rp)
    assert np.array_equal(bufs["col_ptr"].cpu().numpy(), cp)
    for s in range(gm.shape[0]):
        n = rp[s, -1]
        assert np.array_equal(bufs["col_idx"].cpu().numpy()[s, :n], ci[s, :n])
        assert np.array_equal(bufs["row_idx"].cpu().numpy()[s, :n], ri[s, :n])
    return exact, excused


@pytest.mark.parametrize("tau,r_min,r_max", [(0.9, 0, 1), (0.5, 0, 1), (0.99, 0, 1), (2.0, 0, 1),
                                             (0.9, 0.25, 0.25)])
def test_build_mask_tiny_workload(tau, r_min, r_max):
    w = synth.TINY
    qb, kb, _ = synth.make_qkv(w, seed=0)
    p = binding.Params(B=w.B, H=w.H, L=w.L, d=w.d, block=w.block, k_samples=w.k_samples, tau=tau,
                       r_min=r_min, r_max=r_max)
    offs = synth.default_sample_offsets(w.block, w.k_samples)
    _check_build(p, qb, kb, offs, f"tiny tau={tau}")
    if tau == 2.0:
        bufs, _ = _build(p, qb, kb)
        assert bufs["mask"].all()


@pytest.mark.parametrize("grid,n_text,d,block,ks,offs_seed", [
    ((3, 10, 13), 0, 128, 128, 16, None),     # L = 390: tail block of 6 tokens, 1 sample valid
    ((2, 9, 11), 7, 64, 64, 16, None),        # text prefix + grid, L = 205
    ((4, 12, 12), 0, 128, 64, 8, 1),          # random caller-drawn offsets, k = 8
    ((2, 16, 16), 0, 64, 128, 5, 2),          # k = 5
    ((6, 16, 16), 0, 128, 128, 16, 3),        # random offsets, k = 16
])
def test_build_mask_ragged_and_sampled(grid, n_text, d, block, ks, offs_seed):
    w = synth.Workload("t", 1, 3, d, grid, n_text, block, ks)
    print(f"case L={w.L} d={d} block={block} ks={ks}", flush=True)
    qb, kb, _ = synth.make_qkv(w, seed=1, gain=0.7)
    if offs_seed is None:
        offs = synth.default_sample_offsets(block, ks)
        sample = None
    else:
        offs = synth.random_sample_offsets(block, ks, offs_seed)
        sample = offs.tolist()
    p = binding.Params(B=1, H=3, L=w.L, d=d, block=block, k_samples=ks, sample_offsets=sample,
                       tau=0.8)
    _check_build(p, qb, kb, offs, f"L={w.L}")


def test_build_mask_noise_only_inputs_variable_m():
    # nearly flat scores: many rows, m varies, thresholds are crossed with small margins
    shape = (1, 4, 64 * 48, 64)
    qb, kb = synth.make_iid(shape, 5, 0), synth.make_iid(shape, 5, 1)
    p = binding.Params(B=1, H=4, L=shape[2], d=64, block=64, tau=0.3)
    _check_build(p, qb, kb, synth.default_sample_offsets(64, 16), "iid")


def test_build_mask_forced_prefix_rows_and_columns():
    w = synth.Workload("t", 1, 2, 64, (3, 10, 12), 70, 64, 16)
    qb, kb, _ = synth.make_qkv(w, seed=2, gain=0.7)
    offs = synth.default_sample_offsets(64, 16)
    kw = dict(B=1, H=2, L=w.L, d=64, block=64, tau=0.7)
    free, _ = _build(binding.Params(**kw), qb, kb)
    forced, _ = _build(binding.Params(n_prefix_dense=70, **kw), qb, kb)
    fm = free["mask"].cpu().numpy()
    want = oracle.force_prefix(fm, 64, 70)
    assert np.array_equal(forced["mask"].cpu().numpy(), want)
    assert want[:, :2, :].all() and want[:, :, :2].all() and not want.all()


def test_build_mask_without_p_imp_uses_workspace_and_is_deterministic():
    w = synth.TINY
    qb, kb, _ = synth.make_qkv(w, seed=3)
    p = binding.Params(B=w.B, H=w.H, L=w.L, d=w.d, block=w.block, tau=0.9)
    ref, _ = _build(p, qb, kb)
    bufs = binding.alloc_index_lists(p, with_csc=False)
    ws = binding.alloc_workspace(binding.asa_mask_workspace_bytes(p))
    for _ in range(2):
        binding.asa_build_mask(p, util.dev_bf16(qb), util.dev_bf16(kb), bufs["mask"],
                               bufs["row_ptr"], bufs["col_idx"], workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(bufs["mask"], ref["mask"])
        assert torch.equal(bufs["row_ptr"], ref["row_ptr"])
    with pytest.raises(binding.AsaError, match="workspace"):
        binding.asa_build_mask(p, util.dev_bf16(qb), util.dev_bf16(kb), bufs["mask"],
                               bufs["row_ptr"], bufs["col_idx"])


@pytest.mark.parametrize("B,H,L,d,block", [(1, 2, 1024, 64, 64), (1, 2, 1000, 128, 128),
                                            (2, 1, 333, 64, 128), (1, 1, 16384, 64, 64)])
def test_every_token_sampled_gives_the_exact_importance_map(B, H, L, d, block):
    """k = block: no sampling at all, the conceptual definition of Sec. 3.3 Step 1 (soft-max over
    all keys, max-pooled over blocks).  The library computes it on 16-token blocks and max-pools;
    the oracle is its ordinary probe with every offset listed (pinned against the dense soft-max
    in tests/test_oracle_mask.py)."""
    print(f"case B={B} H={H} L={L} d={d} block={block} k={block}", flush=True)
    heads = H if L < 4000 else 1
    qb, kb = (synth.make_iid((B, H, L, d), L + block, s) for s in range(2))
    if L == 1024:
        w = synth.TINY
        qb, kb, _ = synth.make_qkv(w, seed=3)          # video-like, peaked scores
    p = binding.Params(B=B, H=H, L=L, d=d, block=block, k_samples=block, tau=0.9)
    _check_build(p, qb, kb, np.arange(block, dtype=np.int32), f"k=b L={L} block={block}")
    # the seeded build draws "all of them" too
    bufs = binding.alloc_index_lists(p, with_csc=False)
    bufs2 = binding.alloc_index_lists(p, with_csc=False)
    ws = binding.alloc_workspace(binding.asa_mask_seeded_workspace_bytes(p))
    q, k = util.dev_bf16(qb), util.dev_bf16(kb)
    binding.asa_build_mask(p, q, k, bufs["mask"], bufs["row_ptr"], bufs["col_idx"], None, None, None, ws)
    binding.asa_build_mask_seeded(p, 99, q, k, bufs2["mask"], bufs2["row_ptr"], bufs2["col_idx"], None,
                                  None, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(bufs["mask"], bufs2["mask"])
    del heads


def test_every_token_sampled_is_refused_beyond_its_length_limit():
    p = binding.Params(B=1, H=1, L=16385, d=64, block=64, k_samples=64)
    assert binding.asa_mask_workspace_bytes(p) == 0
    p17 = binding.Params(B=1, H=1, L=4096, d=64, block=64, k_samples=17)     # neither <= 16 nor all
    assert binding.asa_mask_workspace_bytes(p17) == 0
