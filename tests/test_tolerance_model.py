"""Where the element-wise allowance of the gradient parity tests comes from (CPU only).

The attention kernels feed the matrix cores bf16 operands, so the probabilities P (for dV) and
dS = P * (dP - Delta) (for dQ, dK) are rounded to 8 significant bits before the second product.
This file redoes the gradient sums of the Tiny workload in fp64 numpy with exactly ONE departure
from the oracle -- that rounding -- and shows, against the oracle itself:

  * the stated plain tolerance (max-abs 2e-2) is below what that rounding alone does on these
    inputs (keys and queries of magnitude up to 9), also on elements of magnitude <= 1;
  * the error of every element stays within 2^-8 times the sum of the absolute values of the
    terms the oracle adds up for it (oracle.attn_bwd(with_mag=True)), which is the allowance
    tests/util.assert_close_bf16 grants on top of the plain figure;
  * Delta taken from a bf16-rounded O is off by several 1e-2 and, times scale * sum_c P_c K_c,
    breaks that allowance: the reason why the library never forms Delta from the bf16 O alone.
"""

import numpy as np

import oracle
from paper_2508_10774_amd import synth
from tests import util


def _bf16(x):
    return synth.round_to_bf16(np.asarray(x, np.float32)).astype(np.float64)


def _tiny_head(h):
    w = synth.TINY
    qb, kb, vb = synth.make_qkv(w, seed=0)
    gb = synth.make_do(w, seed=0)
    f = synth.bf16_bits_to_f32
    mask, _ = oracle.build_mask(f(qb), f(kb), w.block,
                                synth.default_sample_offsets(w.block, w.k_samples), tau=0.9)
    q, k, v, g = (f(x[0, h]) for x in (qb, kb, vb, gb))
    return w, q, k, v, g, mask[0, h]


def _dense_terms(w, q, k, v, g, mask):
    """P, dP, Delta of one head as dense fp64 matrices (the oracle's definitions, vectorised)."""
    q, k, v, g = (x.astype(np.float64) for x in (q, k, v, g))
    keep = np.kron(mask, np.ones((w.block, w.block))).astype(bool)
    sc = oracle.default_scale(w.d)
    s = sc * q @ k.T
    s[~keep] = -np.inf
    e = np.exp(s - s.max(axis=1, keepdims=True))
    p = e / e.sum(axis=1, keepdims=True)
    return sc, p, g @ v.T, (g * (p @ v)).sum(axis=1, keepdims=True), p @ v


def test_bf16_rounding_of_ds_alone_exceeds_the_plain_tolerance_but_not_the_allowance():
    worst_small = 0.0
    for h in range(2):
        w, q, k, v, g, mask = _tiny_head(h)
        wq, wk, wv, mq, mk, mv = oracle.attn_bwd(q, k, v, g, mask, w.block, with_mag=True)
        sc, p, dp, delta, _ = _dense_terms(w, q, k, v, g, mask)
        ds = p * (dp - delta)
        # the vectorised terms are the oracle's (sanity of this file, not a pin of the oracle)
        assert np.abs(sc * ds @ k.astype(np.float64) - wq).max() < 1e-9
        dq = sc * _bf16(ds) @ k.astype(np.float64)
        dk = sc * _bf16(ds).T @ q.astype(np.float64)
        dv = _bf16(p).T @ g.astype(np.float64)
        for got, want, mag in ((dq, wq, mq), (dk, wk, mk), (dv, wv, mv)):
            err = np.abs(got - want)
            assert (err <= util.BF16_UNIT_ROUNDOFF * mag + 1e-12).all()
            small = np.abs(want) <= 1.0
            worst_small = max(worst_small, err[small].max())
    # dQ of head 0: an element of magnitude below 1 is off by more than 2e-2 from this rounding alone
    assert worst_small > util.O_MAX_ABS


def test_delta_from_bf16_o_breaks_the_allowance():
    w, q, k, v, g, mask = _tiny_head(0)
    wq, _, _, mq, _, _ = oracle.attn_bwd(q, k, v, g, mask, w.block, with_mag=True)
    sc, p, dp, delta, o = _dense_terms(w, q, k, v, g, mask)
    delta_bf16 = (g.astype(np.float64) * _bf16(o)).sum(axis=1, keepdims=True)
    assert np.abs(delta_bf16 - delta).max() > 2e-2
    dq = sc * (p * (dp - delta_bf16)) @ k.astype(np.float64)        # everything else exact
    err = np.abs(dq - wq)
    allowance = util.O_MAX_ABS * np.maximum(1.0, np.abs(wq)) + util.BF16_UNIT_ROUNDOFF * mq
    assert (err > allowance).any()
