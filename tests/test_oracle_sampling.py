"""Pins of the seeded sampling oracle: Philox against its published known answers, the draw against
its definition, the per-block importance map against the shared-offset oracle."""

import numpy as np

import oracle
from oracle import random_sampling as rs


def test_philox_known_answers():
    # known-answer vectors distributed with the generator's reference implementation
    assert rs.philox4x32_10((0, 0, 0, 0), (0, 0)) == (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)
    f = 0xffffffff
    assert rs.philox4x32_10((f, f, f, f), (f, f)) == (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)
    assert rs.philox4x32_10((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344),
                            (0xa4093822, 0x299f31d0)) == (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1)


def test_philox_is_a_bijection_of_the_counter_for_a_fixed_key():
    seen = {rs.philox4x32_10((j, 0, 0, 0), (7, 9)) for j in range(2000)}
    assert len(seen) == 2000


def test_block_offsets_are_k_distinct_ascending_positions_and_depend_on_every_input():
    a = rs.block_offsets(42, 3, 5, 128, 16)
    assert a.shape == (16,) and (np.diff(a) > 0).all() and a.min() >= 0 and a.max() < 128
    assert not np.array_equal(a, rs.block_offsets(43, 3, 5, 128, 16))
    assert not np.array_equal(a, rs.block_offsets(42, 4, 5, 128, 16))
    assert not np.array_equal(a, rs.block_offsets(42, 3, 6, 128, 16))
    assert np.array_equal(rs.block_offsets(1 << 40, 0, 0, 64, 64), np.arange(64))     # k = b: everything
    # the sample is the set of the k smallest words
    key = (42, 0)
    words = sorted((rs.philox4x32_10((j, 5, 3, 0), key)[0], j) for j in range(128))
    assert sorted(j for _, j in words[:16]) == a.tolist()


def test_positions_are_used_about_equally_often():
    counts = np.zeros(64)
    for blk in range(400):
        counts[rs.block_offsets(7, 0, blk, 64, 8)] += 1
    expect = 400 * 8 / 64
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert chi2 < 120          # 63 degrees of freedom: mean 63, 120 is beyond the 99.99 % point


def test_per_block_map_with_a_constant_table_equals_the_shared_offset_oracle():
    rng = np.random.default_rng(0)
    L, d, b = 300, 16, 32                       # ragged last block: 12 valid tokens
    q = rng.standard_normal((L, d)).astype(np.float32)
    k = rng.standard_normal((L, d)).astype(np.float32)
    offs = [1, 5, 11, 20, 31]
    Nb = oracle.n_blocks(L, b)
    table = np.tile(np.array(offs, np.uint8), (Nb, 1))
    got = rs.p_imp_table(q, k, b, table)
    want = oracle.p_imp(q, k, b, offs)
    np.testing.assert_allclose(got, want, rtol=2e-7, atol=1e-300)      # the C oracle returns fp32
