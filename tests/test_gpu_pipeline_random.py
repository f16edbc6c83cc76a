"""GPU parity of the whole step on randomly drawn (seeded) shapes and settings.

Each case runs asa_build_mask -> asa_attn_fwd -> asa_attn_bwd through the C ABI on synthetic
video-like tokens and compares every stage with the oracle: the mask row by row (a row may
differ only where the oracle's own scores are closer than the excusal gap), O and LSE on every
row, dQ / dK / dV on every element, with and without the saved low part of O.  The attention
oracle is evaluated on the mask the GPU produced, so that an excused mask row does not hide
behind the attention tolerance."""

import numpy as np
import pytest
import torch

import oracle
from paper_2508_10774_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu


def _draw(seed):
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([64, 128]))
    block = int(rng.choice([64, 128]))
    grid = (int(rng.integers(2, 9)), int(rng.integers(6, 21)), int(rng.integers(6, 21)))
    n_text = int(rng.choice([0, 0, 5, 70]))
    ks = int(rng.choice([16, 16, 8, 3]))
    B, H = (1, int(rng.integers(1, 4))) if rng.random() < 0.7 else (2, 2)
    tau = float(rng.choice([0.5, 0.8, 0.9, 0.97]))
    r_min, r_max = [(0.0, 1.0), (0.1, 0.6), (0.3, 0.3)][int(rng.integers(0, 3))]
    scale = 0.0 if rng.random() < 0.5 else float(rng.uniform(0.05, 0.2))
    return d, block, grid, n_text, ks, B, H, tau, r_min, r_max, scale


@pytest.mark.parametrize("seed", range(8))
def test_mask_forward_backward_chain(seed):
    d, block, grid, n_text, ks, B, H, tau, r_min, r_max, scale = _draw(seed)
    w = synth.Workload("r", B, H, d, grid, n_text, block, ks)
    print(f"case seed={seed} B={B} H={H} L={w.L} d={d} block={block} k={ks} text={n_text} tau={tau} "
          f"r=[{r_min},{r_max}] scale={scale}", flush=True)
    qb, kb, vb = synth.make_qkv(w, seed=seed, gain=0.5)
    gb = synth.make_do(w, seed=seed)
    p = binding.Params(B=B, H=H, L=w.L, d=d, block=block, k_samples=ks, tau=tau, r_min=r_min,
                       r_max=r_max, n_prefix_dense=n_text, scale=scale)
    q, k, v, g = (util.dev_bf16(x) for x in (qb, kb, vb, gb))
    bufs = binding.alloc_index_lists(p)
    pimp = torch.empty((B * H, p.Nb, p.Nb), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(binding.asa_mask_workspace_bytes(p))
    binding.asa_build_mask(p, q, k, bufs["mask"], bufs["row_ptr"], bufs["col_idx"], bufs["col_ptr"],
                           bufs["row_idx"], pimp, ws)
    torch.cuda.synchronize()
    mask_g = bufs["mask"].cpu().numpy().reshape(B * H, p.Nb, p.Nb)
    gp = pimp.cpu().numpy()

    qf, kf, vf, gf = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb, gb))
    offs = synth.default_sample_offsets(block, ks)
    sc = scale if scale else None
    # the GPU mask is the oracle's rule (and forced prefix) applied to the GPU's own scores, bit
    # for bit; the rule on the oracle's scores gives the same rows, or rows excused by score gaps
    self_rule, _ = oracle.mask_rule(gp, tau, r_min, r_max)
    want = oracle.force_prefix(self_rule, block, n_text) if n_text else self_rule
    assert np.array_equal(mask_g, want.reshape(mask_g.shape)), "rule kernel differs on its own scores"
    om, P = oracle.build_mask(qf, kf, block, offs, tau, r_min, r_max, 0, sc)
    exact, excused, failed = util.classify_mask_rows(P, om, self_rule, tau)
    print(f"    mask rows: {exact} exact, {excused} excused, {len(failed)} failed", flush=True)
    assert not failed, failed[:10]
    rp, ci = oracle.csr_from_mask(mask_g)
    assert np.array_equal(bufs["row_ptr"].cpu().numpy(), rp)

    o, lse, o_lo = util.run_fwd(p, q, k, v, bufs, with_lo=True)
    dq, dk, dv = (util.host_f32(x) for x in util.run_bwd(p, q, k, v, o, lse, g, bufs, o_lo=o_lo))
    dq2, dk2, dv2 = (util.host_f32(x) for x in util.run_bwd(p, q, k, v, o, lse, g, bufs))
    of, lf = util.host_f32(o), lse.cpu().numpy().reshape(B, H, w.L)
    for b in range(B):
        for h in range(H):
            m = mask_g[b * H + h]
            wo, wl = oracle.attn_fwd(qf[b, h], kf[b, h], vf[b, h], m, block, sc)
            util.assert_close_bf16(of[b, h], wo, f"O[{b},{h}]")
            fin = np.isfinite(wl)
            assert np.array_equal(fin, np.isfinite(lf[b, h]))
            assert np.abs(lf[b, h][fin] - wl[fin]).max() <= util.LSE_ABS
            wq, wk, wv, mq, mk, mv = oracle.attn_bwd(qf[b, h], kf[b, h], vf[b, h], gf[b, h], m, block,
                                                     sc, with_mag=True)
            for tag, (a_q, a_k, a_v) in (("", (dq, dk, dv)), (" (no o_lo)", (dq2, dk2, dv2))):
                util.assert_close_bf16(a_q[b, h], wq, f"dQ[{b},{h}]" + tag, mq)
                util.assert_close_bf16(a_k[b, h], wk, f"dK[{b},{h}]" + tag, mk)
                util.assert_close_bf16(a_v[b, h], wv, f"dV[{b},{h}]" + tag, mv)
