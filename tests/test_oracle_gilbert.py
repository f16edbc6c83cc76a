"""Pins for the Gilbert-curve token order of the oracle (Sec. 3.3 preprocessing, Alg. 3 step 1).

The paper names the curve and gives no construction, so the pins are what mathematics fixes for
any such curve and what the construction promises: a bijection; unit steps exactly when the
chess-board parity argument allows them; the classical Hilbert curve (textbook bit-twiddling
routine, written out here) on 2^k squares; one contiguous run per aligned sub-cube on 2^k cubes;
and, on the synthetic video tokens, more compact blocks and a lower density at equal tau than
raster order (the reason the paper gives for the step).
"""

import itertools

import numpy as np
import pytest

import oracle
from oracle import gilbert
from paper_2508_10774_amd import synth


def _steps(cells: np.ndarray) -> np.ndarray:
    return np.abs(np.diff(cells, axis=0)).sum(axis=1)


def _is_bijection(cells: np.ndarray, dims) -> bool:
    a, b, c = dims
    if cells.shape != (a * b * c, 3) or (cells < 0).any() or (cells >= np.array(dims)).any():
        return False
    flat = (cells[:, 0] * b + cells[:, 1]) * c + cells[:, 2]
    return np.array_equal(np.sort(flat), np.arange(a * b * c))


def test_every_small_box_is_visited_once_and_in_unit_steps_where_parity_allows():
    N = 9
    n_clean = n_unclean = 0
    for a, b, c in itertools.product(range(1, N + 1), repeat=3):
        cells = gilbert.box_curve(a, b, c)
        assert _is_bijection(cells, (a, b, c)), (a, b, c)
        assert tuple(cells[0]) == (0, 0, 0)
        st = _steps(cells)
        # independent statement of the parity condition: a walk of a*b*c - 1 unit steps from
        # (0,0,0) ends on a cell whose coordinate sum has the parity of a*b*c - 1
        reachable = (a * b * c - 1) % 2 == (a - 1) % 2 and (a > 1 or b * c == 1)
        assert reachable == gilbert.clean(a, b, c)
        if reachable:
            n_clean += 1
            assert (st == 1).all(), (a, b, c)
            assert tuple(cells[-1]) == (a - 1, 0, 0), (a, b, c)
        else:
            n_unclean += 1
            # no unit-step walk can end on that corner: the curve must differ somewhere
            assert tuple(cells[-1]) != (a - 1, 0, 0) or (st != 1).any(), (a, b, c)
    assert n_clean > 300 and n_unclean > 100


def _corner_walk_exists(a: int, b: int, c: int) -> bool:
    """Exhaustive search: is there a walk in unit steps through every cell of the a x b x c box from
    (0, 0, 0) to (a - 1, 0, 0)?"""
    n = a * b * c
    goal = (a - 1, 0, 0)
    seen = {(0, 0, 0)}

    def go(cell, left):
        if left == 0:
            return cell == goal
        if cell == goal:
            return False
        x, y, z = cell
        for nx, ny, nz in ((x + 1, y, z), (x - 1, y, z), (x, y + 1, z), (x, y - 1, z), (x, y, z + 1), (x, y, z - 1)):
            if 0 <= nx < a and 0 <= ny < b and 0 <= nz < c and (nx, ny, nz) not in seen:
                seen.add((nx, ny, nz))
                if go((nx, ny, nz), left - 1):
                    return True
                seen.discard((nx, ny, nz))
        return False

    return go((0, 0, 0), n - 1)


def test_the_parity_condition_is_exactly_when_a_corner_to_corner_walk_exists():
    """Brute force on boxes of up to 24 cells: `clean` (the chess-board argument, a necessary
    condition) is also sufficient there, so the curve's unit steps are all that could be had."""
    n = 0
    for a, b, c in itertools.product(range(1, 7), range(1, 5), range(1, 4)):
        if a * b * c > 24:
            continue
        assert _corner_walk_exists(a, b, c) == gilbert.clean(a, b, c), (a, b, c)
        n += 1
    assert n > 40


def _hilbert_d2xy(n: int, d: int):
    """Textbook conversion of a distance along the Hilbert curve of an n x n square (n = 2^k)
    to coordinates: per level take two bits, rotate/flip the quadrant, add the offset."""
    x = y = 0
    t = d
    s = 1
    while s < n:
        rx = 1 & (t // 2)
        ry = 1 & (t ^ rx)
        if ry == 0:
            if rx == 1:
                x, y = s - 1 - x, s - 1 - y
            x, y = y, x
        x += s * rx
        y += s * ry
        t //= 4
        s *= 2
    return x, y


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32])
def test_power_of_two_square_is_the_classical_hilbert_curve(n):
    cells = gilbert.box_curve(n, n, 1)
    want = np.array([_hilbert_d2xy(n, i) for i in range(n * n)])
    assert np.array_equal(cells[:, :2], want)
    assert (cells[:, 2] == 0).all()


@pytest.mark.parametrize("n", [2, 4, 8, 16])
def test_power_of_two_cube_keeps_every_aligned_subcube_contiguous(n):
    cells = gilbert.box_curve(n, n, n)
    assert (_steps(cells) == 1).all()
    s = 2
    while s <= n:
        runs = cells.reshape(-1, s ** 3, 3)
        lo, hi = runs.min(axis=1), runs.max(axis=1)
        assert (hi - lo + 1 == s).all() and (lo % s == 0).all(), s
        s *= 2


@pytest.mark.parametrize("w", [synth.TINY, synth.WAN, synth.COG, synth.WAN_PADDED], ids=lambda w: w.name)
def test_workload_grids(w):
    order, inverse = gilbert.token_order(w.grid, w.n_text)
    L = w.L
    assert order.dtype == np.int32 and order.shape == (L,)
    assert np.array_equal(np.sort(order), np.arange(L))
    assert np.array_equal(order[:w.n_text], np.arange(w.n_text))
    assert np.array_equal(inverse[order], np.arange(L)) and np.array_equal(order[inverse], np.arange(L))
    T, Y, X = w.grid
    r = order[w.n_text:] - w.n_text
    cells = np.stack([r // (Y * X), (r // X) % Y, r % X], axis=1)
    assert (_steps(cells) == 1).all()
    major, _, _ = gilbert.axis_roles(w.grid)
    assert w.grid[major] % 2 == 0 or all(g % 2 == 1 for g in w.grid)
    # compactness: a block of consecutive tokens spans far fewer rows/frames than in raster order
    nb = (L - w.n_text) // w.block
    runs = cells[:nb * w.block].reshape(nb, w.block, 3)
    extent = (runs.max(axis=1) - runs.min(axis=1) + 1).max(axis=1)
    raster_cells = np.stack(np.unravel_index(np.arange(nb * w.block), w.grid), axis=1).reshape(nb, w.block, 3)
    raster_extent = (raster_cells.max(axis=1) - raster_cells.min(axis=1) + 1).max(axis=1)
    assert extent.mean() < 0.5 * raster_extent.mean()
    # cube root of the block size is the best possible; stay within 3x of it on average
    assert extent.mean() < 3.0 * w.block ** (1.0 / 3.0)


def test_permute_round_trip():
    order, inverse = gilbert.token_order((3, 4, 6), 5)
    x = np.arange(2 * (5 + 72) * 3).reshape(2, 5 + 72, 3)
    y = gilbert.permute_tokens(x, order)
    assert np.array_equal(y[:, 7], x[:, order[7]])
    assert np.array_equal(gilbert.permute_tokens(y, inverse), x)


def test_density_at_equal_tau_is_lower_than_in_raster_order():
    """Sec. 3.3 / Table 'rearrange' ablation: blocks of spatially contiguous tokens concentrate the
    importance mass, so the same tau keeps fewer blocks.  Synthetic video tokens (shared smooth
    field on the grid), 16 x 16 x 16 tokens, block 64."""
    w = synth.Workload("cube", 1, 2, 64, (16, 16, 16), 0, 64, 16)
    qb, kb, _ = synth.make_qkv(w, seed=5)
    q, k = synth.bf16_bits_to_f32(qb), synth.bf16_bits_to_f32(kb)
    offs = synth.default_sample_offsets(w.block, w.k_samples)
    order, _ = gilbert.token_order(w.grid, 0)
    tau = 0.9
    m_raster, _ = oracle.build_mask(q, k, w.block, offs, tau)
    m_curve, _ = oracle.build_mask(gilbert.permute_tokens(q, order), gilbert.permute_tokens(k, order),
                                   w.block, offs, tau)
    assert m_curve.mean() < 0.9 * m_raster.mean(), (m_curve.mean(), m_raster.mean())
