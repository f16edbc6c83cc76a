"""asa_gilbert_order (host code of the library) against the oracle's curve: bit-exact orders.

The function does no GPU work, so these run without a GPU; they call through the C-ABI.
"""

import itertools

import numpy as np
import pytest

from oracle import gilbert
from paper_2508_10774_amd import binding, synth


def _lib_order(grid, n_prefix=0):
    order, inverse = binding.asa_gilbert_order(grid[0], grid[1], grid[2], n_prefix)
    return order.numpy(), inverse.numpy()


def test_every_small_grid_matches_the_oracle():
    n = 0
    for grid in itertools.product(range(1, 8), repeat=3):
        want, want_inv = gilbert.token_order(grid, 0)
        got, got_inv = _lib_order(grid)
        assert np.array_equal(got, want), grid
        assert np.array_equal(got_inv, want_inv), grid
        n += 1
    assert n == 343


@pytest.mark.parametrize("grid,n_prefix", [
    (synth.TINY.grid, 0), (synth.WAN.grid, 0), (synth.COG.grid, synth.COG.n_text), (synth.WAN_PADDED.grid, 0),
    ((1, 30, 52), 0), ((21, 45, 80), 3), ((13, 1, 45), 0), ((1, 1, 1), 2), ((97, 3, 2), 0), ((5, 7, 9), 1),
    ((2, 97, 3), 0), ((1, 1, 100), 0), ((40, 39, 1), 0), ((11, 23, 6), 0)])
def test_workload_and_odd_shaped_grids_match_the_oracle(grid, n_prefix):
    want, want_inv = gilbert.token_order(grid, n_prefix)
    got, got_inv = _lib_order(grid, n_prefix)
    assert np.array_equal(got, want)
    assert np.array_equal(got_inv, want_inv)


def test_random_grids_match_the_oracle_and_step_by_one_cell():
    rng = np.random.default_rng(20250811)
    for _ in range(60):
        grid = tuple(int(x) for x in rng.integers(1, 41, size=3))
        n_prefix = int(rng.integers(0, 4))
        want, want_inv = gilbert.token_order(grid, n_prefix)
        got, got_inv = _lib_order(grid, n_prefix)
        assert np.array_equal(got, want), grid
        assert np.array_equal(got_inv, want_inv), grid
        r = got[n_prefix:].astype(np.int64) - n_prefix
        cells = np.stack([r // (grid[1] * grid[2]), (r // grid[2]) % grid[1], r % grid[2]], axis=1)
        if len(cells) > 1:
            assert (np.abs(np.diff(cells, axis=0)).sum(axis=1) == 1).all(), grid


def test_argument_checks():
    import ctypes
    L = binding.load()
    buf = (ctypes.c_int32 * 16)()
    assert L.asa_gilbert_order(0, 2, 2, 0, buf, None) == -1
    assert L.asa_gilbert_order(2, 2, 2, -1, buf, None) == -1
    assert L.asa_gilbert_order(2, 2, 2, 0, None, None) == -1
    assert L.asa_gilbert_order(2048, 2048, 2048, 0, buf, None) == -2
    assert L.asa_gilbert_order(2, 2, 2, 0, buf, None) == 0      # inverse is optional
    assert sorted(buf[:8]) == list(range(8))
