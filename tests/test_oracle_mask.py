"""Pins for the oracle's mask path (CPU only).

None of these re-type the oracle's formulas in its own shape: they check it against
hand-worked rows, closed forms, a dense soft-max built with numpy, brute-force subset
search in exact rational arithmetic, and invariants of the rule.
"""

import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2508_10774_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))


def _qk(L, d, seed, gain=0.0):
    q = synth.bf16_bits_to_f32(synth.make_iid((L, d), seed, 0))
    k = synth.bf16_bits_to_f32(synth.make_iid((L, d), seed, 1))
    if gain:
        rng = np.random.default_rng(seed + 1000)
        s = np.cumsum(rng.standard_normal((L, d)).astype(np.float32), axis=0)
        s = (s - s.mean()) / s.std()
        q = synth.round_to_bf16(q + gain * s)
        k = synth.round_to_bf16(k + gain * s)
    return q, k


def _dense_softmax(q, k, scale):
    s = (q.astype(np.float64) @ k.astype(np.float64).T) * scale
    s = s.astype(np.float32).astype(np.float64)      # the probe's logits are fp32
    s -= s.max(axis=1, keepdims=True)
    e = np.exp(s)
    return (e / e.sum(axis=1, keepdims=True)).astype(np.float32)


# ---------------------------------------------------------------- sampling

def test_sample_rows_layout_and_padding():
    # Alg. 2 steps 1-3: block t, sample u -> token t*b + off[u]; padded positions drop out
    rows = oracle.sample_rows(L=10, b=4, offs=[0, 3])
    assert rows.tolist() == [0, 3, 4, 7, 8, -1]
    rows = oracle.sample_rows(L=8, b=4, offs=[1, 2])
    assert rows.tolist() == [1, 2, 5, 6]


@pytest.mark.parametrize("offs", [[3, 1], [0, 0], [0, 4], [-1, 2]])
def test_sample_rows_rejects_bad_offsets(offs):
    with pytest.raises(ValueError):
        oracle.sample_rows(L=8, b=4, offs=offs)


# ---------------------------------------------------------------- importance map

@pytest.mark.parametrize("L,b,ks", [(96, 16, 4), (90, 16, 4), (64, 8, 8), (50, 8, 3)])
def test_p_imp_online_form_equals_direct_form(L, b, ks):
    # Alg. 1 (running max / denominator) and Alg. 3 steps 4-5 define the same map
    q, k = _qk(L, 32, seed=L + ks, gain=1.0)
    offs = synth.random_sample_offsets(b, ks, seed=3)
    offs[0] = 0
    a = oracle.p_imp(q, k, b, offs, form="direct")
    o = oracle.p_imp(q, k, b, offs, form="online")
    np.testing.assert_allclose(o, a, rtol=1e-6, atol=0)


@pytest.mark.parametrize("L,b", [(64, 8), (60, 8), (33, 4)])
def test_p_imp_with_every_token_sampled_is_maxpool_of_dense_softmax(L, b):
    # Sec. 3.3 Step 1, the conceptual definition: dense softmax, b x b max-pool
    d = 16
    q, k = _qk(L, d, seed=L, gain=0.5)
    scale = oracle.default_scale(d)
    P = _dense_softmax(q, k, scale)
    Nb = (L + b - 1) // b
    want = np.zeros((Nb, Nb), dtype=np.float32)
    for i in range(Nb):
        for j in range(Nb):
            want[i, j] = P[i * b:(i + 1) * b, j * b:(j + 1) * b].max()
    for form in ("direct", "online"):
        got = oracle.p_imp(q, k, b, np.arange(b), scale, form)
        np.testing.assert_allclose(got, want, rtol=2e-6, atol=0)


def test_p_imp_block_one_is_dense_softmax_matrix():
    L, d = 40, 8
    q, k = _qk(L, d, seed=5, gain=0.3)
    scale = oracle.default_scale(d)
    got = oracle.p_imp(q, k, 1, [0], scale)
    np.testing.assert_allclose(got, _dense_softmax(q, k, scale), rtol=2e-6, atol=0)


def test_p_imp_picks_sampled_tokens_not_their_neighbours():
    # a planted key that only an unsampled token sees must NOT show up; one that a sampled
    # token sees must.  Guards against an off-by-one in t*b + off[u].
    L, d, b = 64, 16, 16
    offs = [2, 9]
    q = np.zeros((L, d), np.float32)
    k = np.zeros((L, d), np.float32)
    q[16 + 9, 0] = 8.0        # block 1, offset 9: sampled
    q[32 + 3, 1] = 8.0        # block 2, offset 3: NOT sampled
    k[48 + 2, 0] = 8.0        # block 3, offset 2: sampled key for channel 0
    k[0 + 9, 1] = 8.0         # block 0, offset 9: sampled key for channel 1
    P = oracle.p_imp(q, k, b, offs, scale=1.0)
    Nk = 4 * 2
    flat = np.float32(1.0 / Nk)
    assert P[1].argmax() == 3 and P[1, 3] > 0.99
    np.testing.assert_allclose(P[2], flat, rtol=1e-6)   # its sampled rows are all-zero queries
    np.testing.assert_allclose(P[0], flat, rtol=1e-6)


def test_p_imp_zero_queries_give_uniform_map():
    L, d, b, ks = 128, 16, 16, 4
    _, k = _qk(L, d, seed=2)
    q = np.zeros((L, d), np.float32)
    for form in ("direct", "online"):
        P = oracle.p_imp(q, k, b, synth.default_sample_offsets(b, ks), form=form)
        assert np.all(P == np.float32(1.0 / (L // b * ks)))


def test_p_imp_bounds_and_row_mass():
    L, d, b, ks = 256, 32, 32, 8
    q, k = _qk(L, d, seed=9, gain=1.0)
    P = oracle.p_imp(q, k, b, synth.default_sample_offsets(b, ks)).astype(np.float64)
    assert np.all(P >= 0) and np.all(P <= 1)
    rs = P.sum(axis=1)
    # every sampled row's probabilities sum to 1: the pooled row holds between one row's
    # average block share (>= 1/k) and the sum of k rows (<= k)
    assert np.all(rs >= 1.0 / ks - 1e-6) and np.all(rs <= ks + 1e-6)


def test_p_imp_scale_argument_is_used():
    L, d, b, ks = 64, 16, 16, 4
    q, k = _qk(L, d, seed=4, gain=0.5)
    offs = synth.default_sample_offsets(b, ks)
    a = oracle.p_imp(q, k, b, offs, scale=0.25)
    c = oracle.p_imp(synth.round_to_bf16(q * 0.5), k, b, offs, scale=0.5)   # same logits
    np.testing.assert_allclose(a, c, rtol=1e-6)
    assert not np.allclose(a, oracle.p_imp(q, k, b, offs, scale=0.5), rtol=1e-3)


def test_p_imp_tail_block_excludes_padding():
    # L = 3 blocks and a bit: the last block has 2 valid tokens, one of them sampled
    b, ks, d = 8, 2, 8
    L = 3 * b + 2
    q, k = _qk(L, d, seed=12, gain=0.5)
    offs = [1, 5]
    got = oracle.p_imp(q, k, b, offs)
    rows = [r for r in oracle.sample_rows(L, b, offs) if r >= 0]
    assert rows == [1, 5, 9, 13, 17, 21, 25]
    P = _dense_softmax(q[rows], k[rows], oracle.default_scale(d))
    blk = [0, 0, 1, 1, 2, 2, 3]
    want = np.zeros((4, 4), np.float32)
    for a, i in enumerate(blk):
        for c, j in enumerate(blk):
            want[i, j] = max(want[i, j], P[a, c])
    np.testing.assert_allclose(got, want, rtol=2e-6)


# ---------------------------------------------------------------- selection rule

def _golden_rows():
    out = []
    with open(os.path.join(HERE, "golden", "rule_examples.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            sc, tau, rmin, rmax, want, _ = [t.strip() for t in line.split("|")]
            out.append((np.array(sc.split(), np.float32), float(tau), float(rmin), float(rmax),
                        np.array(want.split(), np.uint8)))
    return out


@pytest.mark.parametrize("form", ["sort", "orderfree"])
def test_rule_hand_worked_rows(form):
    rows = _golden_rows()
    assert len(rows) >= 12
    for sc, tau, rmin, rmax, want in rows:
        got, m = oracle.mask_rule(sc[None, :], tau, rmin, rmax, form)
        assert got[0].tolist() == want.tolist(), (sc, tau, rmin, rmax)
        assert m[0] == want.sum()


@pytest.mark.parametrize("Nb", [16, 256, 278])
@pytest.mark.parametrize("tau", [0.25, 0.5, 0.9, 0.95, 0.99])
def test_rule_uniform_scores_closed_form(Nb, tau):
    # equal scores: ties go to the lower index, so the row keeps columns 0..m-1 with
    # m = number of r >= 0 with r / Nb < tau  (tau as the fp32 value the rule receives)
    sc = np.full((1, Nb), np.float32(1.0 / 4096), np.float32)
    t32 = Fraction(float(np.float32(tau)))
    m_want = sum(1 for r in range(Nb) if Fraction(r, Nb) < t32)
    for form in ("sort", "orderfree"):
        mask, m = oracle.mask_rule(sc, tau, form=form)
        assert m[0] == m_want
        assert mask[0, :m_want].all() and not mask[0, m_want:].any()


def _brute_force_row(sc, tau32, m_min, m_max):
    """Exact search over all subsets: fewest blocks whose mass reaches tau*T, then the largest
    mass, then the lowest indices; afterwards the clamp adds/removes by the same order."""
    n = len(sc)
    w = [Fraction(float(x)) for x in sc]
    T = sum(w)
    thr = Fraction(float(tau32)) * T
    best = None
    for size in range(1, n + 1):
        cands = []
        for sub in itertools.combinations(range(n), size):
            mass = sum(w[j] for j in sub)
            # the rule keeps adding while the mass BEFORE the next block is below tau*T
            if mass >= thr:
                cands.append((-mass, sub))
        if cands:
            best = min(cands)[1]
            break
    if best is None:
        best = tuple(range(n))
    if thr <= 0:
        best = ()
    order = sorted(range(n), key=lambda j: (-w[j], j))
    m = min(max(len(best), m_min), m_max)
    keep = set(order[:m])
    if m == len(best):
        assert keep == set(best), "top-m by (score desc, index asc) must be the optimal subset"
    return keep


@pytest.mark.parametrize("seed", range(6))
def test_rule_brute_force_small_grids(seed):
    rng = np.random.default_rng(seed)
    for trial in range(40):
        n = int(rng.integers(2, 10))
        if trial % 3 == 0:      # coarse values: many exact ties
            sc = rng.integers(0, 4, size=n).astype(np.float32) / 8
        else:
            sc = rng.random(n, dtype=np.float32) ** 4
        tau = np.float32(rng.choice([0.3, 0.5, 0.75, 0.9, 0.97, 1.0, 1.5]))
        r_min, r_max = [(0.0, 1.0), (0.3, 1.0), (0.0, 0.6), (0.4, 0.4)][trial % 4]
        m_min, m_max = oracle.retention_bounds(n, r_min, r_max)
        want = _brute_force_row(sc, tau, m_min, m_max)
        for form in ("sort", "orderfree"):
            mask, _ = oracle.mask_rule(sc[None], float(tau), r_min, r_max, form)
            assert set(np.nonzero(mask[0])[0].tolist()) == want, (sc, tau, r_min, r_max, form)


def test_retention_bounds_rounding():
    assert oracle.retention_bounds(256, 0.0, 1.0) == (1, 256)
    assert oracle.retention_bounds(256, 0.25, 0.25) == (64, 64)
    assert oracle.retention_bounds(10, 0.25, 0.55) == (3, 5)      # ceil(2.5), floor(5.5)
    assert oracle.retention_bounds(10, 0.0, 0.05) == (1, 1)       # never below one block
    with pytest.raises(ValueError):
        oracle.retention_bounds(10, 0.6, 0.5)


@pytest.mark.parametrize("seed", range(4))
def test_rule_sort_form_equals_orderfree_form(seed):
    rng = np.random.default_rng(100 + seed)
    sc = (rng.random((64, 96), dtype=np.float32) ** 6).astype(np.float32)
    sc[::7] = np.round(sc[::7] * 8) / 8          # ties
    sc[3, 5] = np.nan                             # a NaN score counts as zero
    sc[4] = 0
    for tau, rmin, rmax in [(0.9, 0, 1), (0.5, 0.1, 0.5), (0.99, 0, 0.25), (2.0, 0, 1)]:
        a, ma = oracle.mask_rule(sc, tau, rmin, rmax, "sort")
        c, mc = oracle.mask_rule(sc, tau, rmin, rmax, "orderfree")
        assert np.array_equal(a, c) and np.array_equal(ma, mc)


def test_rule_invariants_and_monotone_in_tau():
    rng = np.random.default_rng(7)
    sc = (rng.random((50, 64), dtype=np.float32) ** 5).astype(np.float32)
    prev = None
    for tau in [0.1, 0.5, 0.8, 0.9, 0.95, 0.99, 1.0]:
        mask, m = oracle.mask_rule(sc, tau)
        assert (m >= 1).all() and np.array_equal(m, mask.sum(axis=1))
        w = sc.astype(np.float64)
        T = w.sum(axis=1)
        kept = (w * mask).sum(axis=1)
        t32 = float(np.float32(tau))
        assert np.all(kept >= t32 * T * (1 - 1e-12))              # reaches the threshold
        weakest = np.where(mask.astype(bool), w, np.inf).min(axis=1)
        assert np.all((kept - weakest < t32 * T * (1 + 1e-12)) | (m == 1))   # and is minimal
        # kept blocks are the largest ones
        assert np.all(np.where(mask.astype(bool), w, np.inf).min(axis=1) >=
                      np.where(mask.astype(bool), -np.inf, w).max(axis=1))
        if prev is not None:
            assert np.all(prev <= mask)                            # nested in tau
        prev = mask


def test_rule_clamps_hold():
    rng = np.random.default_rng(8)
    sc = (rng.random((30, 40), dtype=np.float32) ** 8).astype(np.float32)
    mask, m = oracle.mask_rule(sc, 0.9, r_min=0.2, r_max=0.3)
    assert m.min() >= 8 and m.max() <= 12
    mask, m = oracle.mask_rule(sc, 0.9, r_min=0.25, r_max=0.25)
    assert np.all(m == 10)
    top10 = np.argsort(-sc, axis=1, kind="stable")[:, :10]
    for i in range(30):
        assert set(np.nonzero(mask[i])[0]) == set(top10[i])


def test_force_prefix_rows_and_columns():
    m = np.zeros((2, 6, 6), np.uint8)
    m[:, np.arange(6), np.arange(6)] = 1
    out = oracle.force_prefix(m, b=4, n_prefix=6)      # ceil(6/4) = 2 blocks
    assert out[:, :2, :].all() and out[:, :, :2].all()
    inner = out[:, 2:, 2:]
    assert np.array_equal(inner, m[:, 2:, 2:])
    assert np.array_equal(oracle.force_prefix(m, 4, 0), m)


def test_csr_csc_agree_with_mask():
    mask = synth.random_block_mask(13, 0.3, seed=1, slabs=3)
    rp, ci = oracle.csr_from_mask(mask)
    cp, ri = oracle.csc_from_mask(mask)
    for s in range(3):
        back = np.zeros((13, 13), np.uint8)
        for i in range(13):
            cols = ci[s, rp[s, i]:rp[s, i + 1]]
            assert np.all(np.diff(cols) > 0)
            back[i, cols] = 1
        assert np.array_equal(back, mask[s])
        back[:] = 0
        for j in range(13):
            rows = ri[s, cp[s, j]:cp[s, j + 1]]
            assert np.all(np.diff(rows) > 0)
            back[rows, j] = 1
        assert np.array_equal(back, mask[s])
        assert rp[s, -1] == mask[s].sum() == cp[s, -1]


def test_build_mask_tiny_workload_end_to_end():
    w = synth.TINY
    qb, kb, _ = synth.make_qkv(w, seed=0)
    q = synth.bf16_bits_to_f32(qb)
    k = synth.bf16_bits_to_f32(kb)
    offs = synth.default_sample_offsets(w.block, w.k_samples)
    mask, P = oracle.build_mask(q, k, w.block, offs, tau=0.9)
    assert mask.shape == (1, 2, 16, 16) and P.shape == (1, 2, 16, 16)
    assert (mask.sum(axis=-1) >= 1).all()
    # smooth field shared by Q and K (blurred across the 4 frames too): the best-matching key
    # block covers the same grid rows as the query block, in some frame
    assert (P.argmax(axis=-1) % 4 == np.arange(16) % 4).mean() > 0.75
    full, _ = oracle.build_mask(q, k, w.block, offs, tau=2.0)
    assert full.all()
