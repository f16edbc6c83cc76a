"""Helpers shared by the GPU parity tests (no method arithmetic here)."""

import numpy as np
import torch

from paper_2508_10774_amd import binding, synth

O_MAX_ABS = 2e-2      # max-abs tolerance on O, dQ, dK, dV for bf16 inputs
O_MEAN_ABS = 2e-3     # mean-abs tolerance
LSE_ABS = 1e-3


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bits -> torch.bfloat16 tensor on the GPU (same bits)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.view(torch.bfloat16).cuda()


def host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def lists_from_mask(p: binding.Params, mask_np: np.ndarray, with_csc=True):
    """Upload a [S, Nb, Nb] uint8 mask and build its index lists with the library."""
    bufs = binding.alloc_index_lists(p, with_csc=with_csc)
    bufs["mask"].copy_(torch.from_numpy(np.ascontiguousarray(mask_np.reshape(bufs["mask"].shape))))
    binding.asa_csr_from_mask(p, bufs["mask"], bufs["row_ptr"], bufs["col_idx"],
                              bufs.get("col_ptr"), bufs.get("row_idx"))
    return bufs


def run_fwd(p: binding.Params, q, k, v, bufs, with_lo=False):
    o = torch.empty((p.B, p.H, p.L, p.d), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((p.B * p.H, p.L), dtype=torch.float32, device="cuda")
    o_lo = torch.empty_like(o) if with_lo else None
    ws = binding.alloc_workspace(binding.asa_fwd_workspace_bytes(p))
    binding.asa_attn_fwd(p, q, k, v, bufs["row_ptr"], bufs["col_idx"], o, lse, ws, o_lo=o_lo)
    torch.cuda.synchronize()
    return (o, lse, o_lo) if with_lo else (o, lse)


BF16_UNIT_ROUNDOFF = 2.0 ** -8   # largest relative error of rounding to bf16 (8 significant bits)


def assert_close_bf16(got: np.ndarray, want: np.ndarray, what: str, mag: np.ndarray = None,
                      max_abs=O_MAX_ABS, mean_abs=O_MEAN_ABS):
    """The stated tolerance: max |got - want| <= 2e-2 and mean |got - want| <= 2e-3.

    mag is None (O, and every tensor of a test that passes no magnitudes): exactly that, on
    every element.

    mag given (gradients): the element-wise allowance is
        max_abs * max(1, |want|)  +  2^-8 * mag
    with mag[r, x] the sum of the absolute values of the terms that the oracle adds up for
    that element (oracle.attn_bwd(..., with_mag=True)); the mean-abs criterion stays plain.
    Where the allowance comes from: the matrix cores take bf16 operands, so P (for dV) and dS
    (for dQ, dK) are rounded to 8 significant bits before they are multiplied with dO, K, Q,
    each term of the sum picks up a relative error of up to 2^-8, and the sum of |terms| is
    what bounds the result's error, however much the terms cancel; the result itself is
    stored in bf16 (2^-8 |want| < max_abs |want|).  An element of magnitude <= 1 whose terms
    are small gets the plain 2e-2.  That the plain figure cannot hold where mag is large is
    shown on the CPU in tests/test_tolerance_model.py (rounding dS alone, everything else
    exact, already exceeds it).

    Prints the plain maximum and mean, the number of elements beyond the plain figure and the
    largest error relative to the allowance; returns (plain max, plain mean).
    """
    got = got.astype(np.float64)
    want = want.astype(np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    err = np.abs(got - want)
    if mag is None:
        bound = np.full_like(err, max_abs)
    else:
        bound = max_abs * np.maximum(1.0, np.abs(want)) + BF16_UNIT_ROUNDOFF * mag.astype(np.float64)
    rel = err / bound
    over_plain = int((err > max_abs).sum())
    print(f"    {what}: max-abs {err.max():.3e} mean-abs {err.mean():.3e} | beyond {max_abs:g}: "
          f"{over_plain} of {err.size} | max err/allowance {rel.max():.3f}", flush=True)
    i = np.unravel_index(np.argmax(rel), rel.shape)
    assert rel.max() <= 1.0, (f"{what}: |err| {err[i]:.3e} > allowance {bound[i]:.3e} at {i} "
                              f"(want {want[i]:.4f})")
    assert err.mean() <= mean_abs, f"{what}: mean-abs {err.mean():.3e} > {mean_abs}"
    return float(err.max()), float(err.mean())


# ---------------------------------------------------------------------------
# mask parity accounting
# ---------------------------------------------------------------------------

SCORE_GAP = 1e-6   # normalised-score gap below which a mask disagreement is excused


def classify_mask_rows(P, mask_o, mask_g, tau, gap=SCORE_GAP):
    """Compare GPU and oracle masks row by row (no forced prefix in either).

    P: oracle importance map [..., Nb] fp32.  A row whose masks differ is *excused* only if
    the difference is explained by oracle scores that are closer than `gap` (normalised by
    the row sum): (a) a different m needs every cumulative normalised score between the two
    m's to lie within `gap` of tau; (b) blocks swapped at equal m need normalised scores
    within `gap` of each other.  Returns (exact, excused, failed) row counts and the list of
    failed rows.
    """
    Nb = P.shape[-1]
    P2 = np.nan_to_num(P.reshape(-1, Nb).astype(np.float64), nan=0.0)
    mo = mask_o.reshape(-1, Nb).astype(bool)
    mg = mask_g.reshape(-1, Nb).astype(bool)
    t32 = float(np.float32(tau))
    exact = excused = 0
    failed = []
    for r in np.nonzero((mo != mg).any(axis=1))[0]:
        w = P2[r]
        T = w.sum() or 1.0
        order = np.lexsort((np.arange(Nb), -w))
        s = w[order] / T
        cum = np.concatenate([[0.0], np.cumsum(s)])
        m_o, m_g = int(mo[r].sum()), int(mg[r].sum())
        ok = True
        if m_o != m_g:
            lo, hi = sorted((m_o, m_g))
            ok = all(abs(cum[x] - t32) < gap for x in range(lo, hi))
        if ok:
            top_g = np.zeros(Nb, bool)
            top_g[order[:m_g]] = True
            diff = np.nonzero(top_g != mg[r])[0]
            if len(diff):
                sc = w[diff] / T
                ok = (sc.max() - sc.min()) < gap
        if ok:
            excused += 1
        else:
            failed.append(int(r))
    exact = mo.shape[0] - excused - len(failed)
    return exact, excused, failed


def run_bwd(p: binding.Params, q, k, v, o, lse, d_o, bufs, o_lo=None):
    dq = torch.full_like(q, float("nan"))
    dk = torch.full_like(k, float("nan"))
    dv = torch.full_like(v, float("nan"))
    ws = binding.alloc_workspace(binding.asa_bwd_workspace_bytes(p))
    binding.asa_attn_bwd(p, q, k, v, o, d_o, lse, bufs["row_ptr"], bufs["col_idx"],
                         bufs["col_ptr"], bufs["row_idx"], dq, dk, dv, ws, o_lo=o_lo)
    torch.cuda.synchronize()
    return dq, dk, dv
