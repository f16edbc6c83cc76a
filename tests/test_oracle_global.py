"""Pins of the ASA_G oracle (global tokens, Sec. 3.3) against what the mathematics fixes."""

import math

import numpy as np
import torch

import oracle
from oracle import global_tokens as og


def _rand(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


def _bf16(x):
    return torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()


def test_pool_is_the_window_mean_and_rounds_to_bf16_nearest_even():
    x = _bf16(_rand((10, 4), 0))
    m, cnt = og.pool(x, 4, exact_pool=True)
    assert cnt.tolist() == [4, 4, 2]
    np.testing.assert_allclose(m[0], x[:4].astype(np.float64).mean(0), rtol=0, atol=1e-15)
    np.testing.assert_allclose(m[2], x[8:].astype(np.float64).mean(0), rtol=0, atol=1e-15)
    r, _ = og.pool(x, 4)
    want = torch.from_numpy(m).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(r, want)          # torch's bf16 cast is round-to-nearest-even
    # exact ties go to the even mantissa: 1 + 2^-8 lies halfway between bf16(1) and bf16(1 + 2^-7)
    tie = np.array([[1.0 + 2.0 ** -8], [1.0 + 3 * 2.0 ** -8]])
    np.testing.assert_array_equal(og._round_bf16(tie)[:, 0], [1.0, 1.0 + 2.0 ** -6])


def test_window_of_one_doubles_every_key_and_changes_nothing_but_lse():
    # n = 1: the pooled tokens are the tokens themselves with bias ln 1 = 0.  With the full mask
    # every key then appears twice with equal weight: same O as plain attention, LSE + ln 2.
    L, d, b = 96, 16, 32
    q, k, v = (_bf16(_rand((L, d), s)) for s in range(3))
    mask = np.ones((3, 3), np.uint8)
    o, lse = og.attn_fwd_g(q, k, v, mask, b, 1)
    o0, lse0 = oracle.attn_fwd(q, k, v, mask, b)
    np.testing.assert_allclose(o, o0, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, lse0 + math.log(2.0), rtol=0, atol=1e-12)


def test_constant_keys_inside_windows_make_global_tokens_equal_dense_attention():
    # If all keys of a window are equal, sum_{i in w} exp(q.k_i) v_i = n exp(q.kbar_w) vbar_w:
    # with an EMPTY block mask the ln(n) bias makes ASA_G reproduce dense attention exactly.
    L, d, b, n = 128, 8, 32, 16
    q = _bf16(_rand((L, d), 1))
    kw = _bf16(_rand((L // n, d), 2))
    k = np.repeat(kw, n, axis=0)
    v = np.random.default_rng(3).integers(-8, 9, size=(L, d)).astype(np.float32)   # means exact in bf16
    # window means of small integers over 16 tokens are multiples of 1/16 below 2^8: exact in bf16
    empty = np.zeros((4, 4), np.uint8)
    o, lse = og.attn_fwd_g(q, k, v, empty, b, n)
    dense = np.ones((4, 4), np.uint8)
    o0, lse0 = oracle.attn_fwd(q, k, v, dense, b)
    np.testing.assert_allclose(o, o0, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, lse0, rtol=0, atol=1e-12)


def test_masked_part_alone_is_standard_asa_when_global_tokens_are_far_away():
    # pooled keys with a hugely negative score contribute nothing: O and LSE fall back to ASA's
    L, d, b, n = 96, 8, 32, 32
    q = np.abs(_bf16(_rand((L, d), 4))) + 1.0
    k = _bf16(_rand((L, d), 5))
    k[:, 0] = np.where(np.arange(L) % 2 == 0, 40.0, -40.0)   # window means ~0 in channel 0 ...
    v = _bf16(_rand((L, d), 6))
    mask = np.array([[1, 0, 1], [0, 1, 0], [1, 1, 1]], np.uint8)
    k2 = k.copy()
    # ... so shift every key far along -q's positive orthant only in the pooled copy: emulate by scale
    o, lse = og.attn_fwd_g(q, k2, v, mask, b, n, scale=1.0)
    o0, lse0 = oracle.attn_fwd(q, k2, v, mask, b, 1.0)
    # the kept even-index keys score +40 q_0 ~ >= 40, pooled keys ~0: weight <= n e^{-40}
    np.testing.assert_allclose(o, o0, rtol=0, atol=1e-9)
    np.testing.assert_allclose(lse, lse0, rtol=0, atol=1e-9)


def test_rows_are_convex_combinations_and_lse_matches_brute_force():
    L, d, b, n = 70, 8, 16, 8          # ragged last block (6 valid) and ragged last window (6 valid)
    q, k, v = (_bf16(_rand((L, d), s + 10)) for s in range(3))
    mask = (np.random.default_rng(0).random((5, 5)) < 0.5).astype(np.uint8)
    o, lse = og.attn_fwd_g(q, k, v, mask, b, n)
    kg, cnt = og.pool(k, n)
    vg, _ = og.pool(v, n)
    assert cnt[-1] == 6
    sc = og.default_scale(d)
    for r in (0, 17, 69):
        tot, acc = 0.0, np.zeros(d)
        for j in range(L):
            if mask[r // b, j // b]:
                w = math.exp(sc * float(np.dot(q[r].astype(np.float64), k[j].astype(np.float64))))
                tot += w
                acc += w * v[j].astype(np.float64)
        for w_i in range(kg.shape[0]):
            w = n * math.exp(sc * float(np.dot(q[r].astype(np.float64), kg[w_i])))
            tot += w
            acc += w * vg[w_i]
        np.testing.assert_allclose(o[r], acc / tot, rtol=1e-12, atol=1e-12)
        assert abs(lse[r] - math.log(tot)) < 1e-12


def test_gradients_match_central_finite_differences():
    L, d, b, n = 40, 4, 8, 4
    rng = np.random.default_rng(7)
    q, k, v, g = (rng.standard_normal((L, d)) for _ in range(4))
    mask = (rng.random((5, 5)) < 0.5).astype(np.uint8)
    mask[2, :] = 0                      # a query block that sees global tokens only
    dq, dk, dv = og.attn_bwd_g(q, k, v, g, mask, b, n, exact_pool=True)

    def loss(q_, k_, v_):
        o, _ = og.attn_fwd_g(q_, k_, v_, mask, b, n, exact_pool=True)
        return float((o * g).sum())

    h = 1e-5
    for name, grad, idx in (("q", dq, (3, 1)), ("q", dq, (17, 0)), ("k", dk, (9, 2)), ("k", dk, (39, 3)),
                            ("v", dv, (0, 0)), ("v", dv, (22, 1))):
        args = {"q": q.copy(), "k": k.copy(), "v": v.copy()}
        args[name][idx] += h
        up = loss(args["q"], args["k"], args["v"])
        args[name][idx] -= 2 * h
        dn = loss(args["q"], args["k"], args["v"])
        fd = (up - dn) / (2 * h)
        assert abs(fd - grad[idx]) < 1e-7 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])


def test_gradient_of_the_pooled_part_is_spread_evenly_over_the_window():
    # empty mask: K and V matter only through their window means, so tokens of one window get
    # identical gradients, each 1 / count of the window's
    L, d, b, n = 24, 4, 8, 8
    rng = np.random.default_rng(8)
    q, k, v, g = (rng.standard_normal((L, d)) for _ in range(4))
    dq, dk, dv = og.attn_bwd_g(q, k, v, g, np.zeros((3, 3), np.uint8), b, n, exact_pool=True)
    for w in range(3):
        for grad in (dk, dv):
            blk = grad[w * n:(w + 1) * n]
            np.testing.assert_allclose(blk, np.broadcast_to(blk[0], blk.shape), rtol=0, atol=1e-15)
