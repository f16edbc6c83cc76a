"""Pins for the oracle's masked attention and its gradients (CPU only).

Checked against library routines (torch scaled_dot_product_attention and autograd in fp64),
closed forms, Richardson-extrapolated finite differences and conservation identities.
"""

import numpy as np
import pytest
import torch

import oracle
from paper_2508_10774_amd import synth


def _qkv(L, d, seed, n=3):
    return [synth.bf16_bits_to_f32(synth.make_iid((L, d), seed, s)) for s in range(n)]


def _token_mask(mask, L, b):
    return np.repeat(np.repeat(mask.astype(bool), b, axis=0), b, axis=1)[:L, :L]


def _torch_attn(q, k, v, mask, b, scale):
    L = q.shape[0]
    tm = torch.from_numpy(_token_mask(mask, L, b))
    tq, tk, tv = (torch.from_numpy(x.astype(np.float64)) for x in (q, k, v))
    bias = torch.zeros(L, L, dtype=torch.float64).masked_fill(~tm, float("-inf"))
    o = torch.nn.functional.scaled_dot_product_attention(tq[None], tk[None], tv[None],
                                                         attn_mask=bias[None], scale=scale)
    return o[0].numpy()


@pytest.mark.parametrize("L,d,b", [(128, 32, 16), (100, 16, 16), (77, 64, 32)])
def test_all_blocks_kept_is_dense_attention(L, d, b):
    q, k, v = _qkv(L, d, seed=L)
    Nb = (L + b - 1) // b
    mask = np.ones((Nb, Nb), np.uint8)
    o, lse = oracle.attn_fwd(q, k, v, mask, b)
    scale = oracle.default_scale(d)
    want = torch.nn.functional.scaled_dot_product_attention(
        *(torch.from_numpy(x.astype(np.float64))[None] for x in (q, k, v)), scale=scale)[0].numpy()
    np.testing.assert_allclose(o, want, rtol=1e-10, atol=1e-12)
    # and the textbook triple product, written with numpy
    s = (q.astype(np.float64) @ k.astype(np.float64).T) * scale
    np.testing.assert_allclose(lse, np.log(np.exp(s).sum(axis=1)), rtol=1e-12)
    p = np.exp(s - lse[:, None])
    np.testing.assert_allclose(o, p @ v.astype(np.float64), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("L,d,b,dens", [(128, 32, 16, 0.3), (120, 16, 16, 0.5), (200, 64, 64, 0.5)])
def test_block_mask_equals_dense_attention_with_minus_inf_bias(L, d, b, dens):
    q, k, v = _qkv(L, d, seed=L + 1)
    Nb = (L + b - 1) // b
    mask = synth.random_block_mask(Nb, dens, seed=L)[0]
    o, _ = oracle.attn_fwd(q, k, v, mask, b)
    want = _torch_attn(q, k, v, mask, b, oracle.default_scale(d))
    np.testing.assert_allclose(o, want, rtol=1e-10, atol=1e-12)


def test_constant_and_one_hot_values():
    L, d, b = 96, 16, 16
    q, k, _ = _qkv(L, d, seed=3)
    mask = synth.random_block_mask(6, 0.4, seed=2)[0]
    o, _ = oracle.attn_fwd(q, k, np.ones((L, d), np.float32), mask, b)
    np.testing.assert_allclose(o, 1.0, rtol=1e-12)
    # V = identity-like: channel x collects the probability of key x
    v = np.zeros((L, d), np.float32)
    v[np.arange(L), np.arange(L) % d] = 1.0
    o, _ = oracle.attn_fwd(q, k, v, mask, b)
    np.testing.assert_allclose(o.sum(axis=1), 1.0, rtol=1e-12)
    assert (o >= 0).all()
    # a dropped block contributes nothing: with exactly one key block kept, V constant per
    # block, the output is that block's constant
    single = np.zeros((6, 6), np.uint8)
    single[np.arange(6), (np.arange(6) + 2) % 6] = 1
    vb = np.repeat(np.arange(6, dtype=np.float32)[:, None], b, axis=0) * np.ones((1, d), np.float32)
    o, _ = oracle.attn_fwd(q, k, vb, single, b)
    want = np.repeat((np.arange(6) + 2) % 6, b).astype(np.float64)
    np.testing.assert_allclose(o, want[:, None] * np.ones((1, d)), rtol=1e-12)


def test_qblocks_subset_matches_full_and_marks_rest_nan():
    L, d, b = 112, 16, 16
    q, k, v = _qkv(L, d, seed=6)
    mask = synth.random_block_mask(7, 0.4, seed=6)[0]
    full, lse_full = oracle.attn_fwd(q, k, v, mask, b)
    part, lse = oracle.attn_fwd(q, k, v, mask, b, qblocks=[1, 6])
    rows = np.r_[16:32, 96:112]
    assert np.array_equal(part[rows], full[rows]) and np.array_equal(lse[rows], lse_full[rows])
    rest = np.setdiff1d(np.arange(L), rows)
    assert np.isnan(part[rest]).all() and np.isnan(lse[rest]).all()


def test_scale_argument():
    L, d, b = 64, 16, 16
    q, k, v = _qkv(L, d, seed=8)
    mask = np.ones((4, 4), np.uint8)
    a, la = oracle.attn_fwd(q, k, v, mask, b, scale=0.125)
    c, lc = oracle.attn_fwd(synth.round_to_bf16(2 * q), k, v, mask, b, scale=0.0625)
    np.testing.assert_allclose(a, c, rtol=1e-12)
    np.testing.assert_allclose(la, lc, rtol=1e-12)


# ---------------------------------------------------------------- gradients

def _torch_grads(q, k, v, do, mask, b, scale):
    L = q.shape[0]
    tm = torch.from_numpy(_token_mask(mask, L, b))
    tq, tk, tv = (torch.from_numpy(x.astype(np.float64)).requires_grad_(True) for x in (q, k, v))
    s = (tq @ tk.T) * scale
    s = s.masked_fill(~tm, float("-inf"))
    o = torch.softmax(s, dim=-1) @ tv
    (o * torch.from_numpy(do.astype(np.float64))).sum().backward()
    return tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy()


@pytest.mark.parametrize("L,d,b,dens", [(96, 16, 16, 0.4), (100, 32, 16, 0.5), (128, 64, 64, 1.0)])
def test_gradients_equal_autograd_fp64(L, d, b, dens):
    q, k, v, do = _qkv(L, d, seed=L + 5, n=4)
    Nb = (L + b - 1) // b
    mask = synth.random_block_mask(Nb, dens, seed=L)[0] if dens < 1 else np.ones((Nb, Nb), np.uint8)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, mask, b)
    wq, wk, wv = _torch_grads(q, k, v, do, mask, b, oracle.default_scale(d))
    np.testing.assert_allclose(dq, wq, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dk, wk, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dv, wv, rtol=1e-9, atol=1e-11)


def test_gradients_finite_differences():
    L, d, b = 48, 8, 8
    q, k, v, do = _qkv(L, d, seed=21, n=4)
    mask = synth.random_block_mask(6, 0.5, seed=3)[0]
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, mask, b)

    def loss(qq, kk, vv):
        o, _ = oracle.attn_fwd(qq, kk, vv, mask, b)
        return float((o * do.astype(np.float64)).sum())

    def central(which, idx, h):
        args = [q.copy(), k.copy(), v.copy()]
        args[which][idx] += np.float32(h)
        up = loss(*args)
        args[which][idx] -= np.float32(2 * h)
        return (up - loss(*args)) / (2 * h)

    rng = np.random.default_rng(0)
    for which, g in enumerate((dq, dk, dv)):
        for _ in range(6):
            idx = (int(rng.integers(L)), int(rng.integers(d)))
            # steps are powers of two, exact in fp32 next to bf16-valued inputs;
            # Richardson removes the h^2 term
            fd = (4 * central(which, idx, 2.0 ** -9) - central(which, idx, 2.0 ** -8)) / 3
            assert abs(fd - g[idx]) <= 1e-7 * max(1.0, abs(g[idx])), (which, idx, fd, g[idx])


def test_gradient_identities():
    L, d, b = 96, 16, 16
    q, k, v, do = _qkv(L, d, seed=31, n=4)
    mask = synth.random_block_mask(6, 0.5, seed=4)[0]
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, mask, b)
    q64, k64 = q.astype(np.float64), k.astype(np.float64)
    # rescaling Q by a and K by 1/a leaves the output unchanged
    assert abs((q64 * dq).sum() - (k64 * dk).sum()) < 1e-9
    # softmax rows sum to one: dV collects all of dO
    tm = _token_mask(mask, L, b)
    reached = tm.any(axis=0)
    assert reached.all()
    np.testing.assert_allclose(dv.sum(axis=0), do.astype(np.float64).sum(axis=0), rtol=1e-10)
    # shifting every key of one row's kept set by a common vector changes nothing when all
    # blocks are kept
    full = np.ones((6, 6), np.uint8)
    _, dk_full, _ = oracle.attn_bwd(q, k, v, do, full, b)
    np.testing.assert_allclose(dk_full.sum(axis=0), 0.0, atol=1e-10)


def test_bwd_block_subsets_match_full():
    L, d, b = 96, 16, 16
    q, k, v, do = _qkv(L, d, seed=41, n=4)
    mask = synth.random_block_mask(6, 0.5, seed=5)[0]
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, mask, b)
    pq, pk, pv = oracle.attn_bwd(q, k, v, do, mask, b, qblocks=[2], kblocks=[0, 5])
    np.testing.assert_allclose(pq[32:48], dq[32:48], rtol=1e-13)
    assert np.isnan(pq[:32]).all() and np.isnan(pq[48:]).all()
    for sl in (slice(0, 16), slice(80, 96)):
        np.testing.assert_allclose(pk[sl], dk[sl], rtol=1e-13)
        np.testing.assert_allclose(pv[sl], dv[sl], rtol=1e-13)
    assert np.isnan(pk[16:80]).all()


def test_tail_rows_and_columns():
    # L not a multiple of b: keys past L never contribute, rows past L do not exist
    L, d, b = 90, 16, 16
    q, k, v, do = _qkv(L, d, seed=51, n=4)
    mask = synth.random_block_mask(6, 0.5, seed=6)[0]
    mask[:, 5] = 1
    o, lse = oracle.attn_fwd(q, k, v, mask, b)
    want = _torch_attn(q, k, v, mask, b, oracle.default_scale(d))
    np.testing.assert_allclose(o, want, rtol=1e-10, atol=1e-12)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, mask, b)
    wq, wk, wv = _torch_grads(q, k, v, do, mask, b, oracle.default_scale(d))
    np.testing.assert_allclose(dq, wq, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dk, wk, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dv, wv, rtol=1e-9, atol=1e-11)
