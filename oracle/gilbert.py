"""Token order along a generalised Hilbert ("Gilbert") curve through a T x Y x X grid.

TEST INFRASTRUCTURE ONLY: a plain, slow reference that the tests, the smoke check and the
benchmark's cpu_baseline leg compare the library with.  Nothing of the product imports it.

What it follows.  Sec. 3.3 ("Preprocessing and Importance Estimation") and Alg. 3 step 1 rearrange
the video tokens along a Gilbert space-filling curve before they are cut into blocks, so that a
block holds tokens that are neighbours in the video; the paper names the curve and cites it, it
does not define it.  The construction below is therefore this build's own reading, derived from
three requirements: (1) every cell of the grid is visited once; (2) consecutive cells are grid
neighbours (one unit step) whenever parity allows it at all; (3) on a 2^k square it IS the
classical Hilbert curve, and on a 2^k cube every aligned 2^j sub-cube is one contiguous run.

Construction.  walk(p, A, B, C) visits the box spanned from corner p by the axis-parallel vectors
A (major), B, C (lengths a, b, c), starts at p and ends at the far end of the major edge,
p + (a-1) A^.  Colouring the cells like a chess board shows when unit steps can do that: the
walk makes a*b*c - 1 colour changes and must arrive on the colour of p + (a-1) A^, so it needs
    clean(a; b, c):  a even, or b and c both odd            (and b = c = 1 if a = 1).
A box is cut in one of four ways; each piece is a box of the same kind and the end of a piece is
a grid neighbour of the start of the next one:
    W   two pieces along the major axis               (a1; b, c) (a2; b, c)
    UB  a "U" in the A-B plane                         (b1; a1, c) (a; b2, c) (b1; a2, c)
    UC  the same in the A-C plane                      (c1; a1, b) (a; c2, b) (c1; a2, b)
    3D  five pieces (the Hilbert cube step)            (b1; c1, a1) (c; a1, b2) (a; b1, c2)
                                                       (c; b2, a2) (b1; a2, c1)
with a = a1 + a2 etc.  The cut is chosen by shape: a minor axis is "long" if 3 * length >=
2 * (longest of the three) and length >= 2; both long -> 3D, only b -> UB, only c -> UC, none ->
W; the other kinds follow in the order W, UB, UC, 3D if the preferred one has no admissible cut.
Cut positions are tried nearest the middle first (the 4 values x of 1..n-1 with the smallest
(|2x - n|, x)), the first axis of the kind's parameter list varying slowest; the first cut
whose pieces are all `clean` is taken.  (If there is none - only below a box that was not clean
itself - the cut with the fewest unclean pieces is taken and the curve has a longer step there.)
A box with a = 1 that is not a single cell cannot end where it starts: it is walked with its
longest side as major axis.

Top level: the major axis is the longest axis of even length (any axis if all are odd: longest),
ties to the earlier of (T, Y, X); B is the longer of the other two (tie: the earlier).  With that
choice the whole grid is always `clean`.
"""

from __future__ import annotations

import itertools
import sys
from typing import List, Sequence, Tuple

import numpy as np

Vec = Tuple[int, int, int]


def clean(a: int, b: int, c: int) -> bool:
    """Necessary condition for a unit-step walk of an a x b x c box from a corner to the far end
    of its a-edge (chess-board colouring)."""
    if a == 1:
        return b == 1 and c == 1
    return a % 2 == 0 or (b % 2 == 1 and c % 2 == 1)


def cut_positions(n: int) -> List[int]:
    """Up to four cut positions of an axis of length n, nearest the middle first."""
    return sorted(range(1, n), key=lambda x: (abs(2 * x - n), x))[:4]


def _pieces(kind: str, a: int, b: int, c: int, s: Sequence[int]) -> List[Tuple[int, int, int]]:
    if kind == "W":
        return [(s[0], b, c), (a - s[0], b, c)]
    if kind == "UB":
        a1, b1 = s
        return [(b1, a1, c), (a, b - b1, c), (b1, a - a1, c)]
    if kind == "UC":
        a1, c1 = s
        return [(c1, a1, b), (a, c - c1, b), (c1, a - a1, b)]
    a1, b1, c1 = s
    return [(b1, c1, a1), (c, a1, b - b1), (a, b1, c - c1), (c, b - b1, a - a1), (b1, a - a1, c1)]


def _cuts(kind: str, a: int, b: int, c: int):
    if kind == "W":
        return itertools.product(cut_positions(a))
    if kind == "UB":
        return itertools.product(cut_positions(a), cut_positions(b))
    if kind == "UC":
        return itertools.product(cut_positions(a), cut_positions(c))
    return itertools.product(cut_positions(a), cut_positions(b), cut_positions(c))


def choose_cut(a: int, b: int, c: int):
    longest = max(a, b, c)
    b_long = b >= 2 and 3 * b >= 2 * longest
    c_long = c >= 2 and 3 * c >= 2 * longest
    first = "3D" if (b_long and c_long) else "UB" if b_long else "UC" if c_long else "W"
    fallback = None
    for kind in [first] + [k for k in ("W", "UB", "UC", "3D") if k != first]:
        for s in _cuts(kind, a, b, c):
            unclean = sum(not clean(*piece) for piece in _pieces(kind, a, b, c, s))
            if unclean == 0:
                return kind, s
            if fallback is None or unclean < fallback[0]:
                fallback = (unclean, kind, s)
    return fallback[1], fallback[2]


def _scaled(u: Vec, k: int) -> Vec:
    return (u[0] * k, u[1] * k, u[2] * k)


def _sum(*vs: Vec) -> Vec:
    return (sum(v[0] for v in vs), sum(v[1] for v in vs), sum(v[2] for v in vs))


def _length_and_direction(v: Vec):
    n = abs(v[0]) + abs(v[1]) + abs(v[2])   # axis-parallel: one non-zero component
    return n, tuple((x > 0) - (x < 0) for x in v)


def walk(p: Vec, A: Vec, B: Vec, C: Vec, out: List[Vec]) -> None:
    a, ua = _length_and_direction(A)
    b, ub = _length_and_direction(B)
    c, uc = _length_and_direction(C)
    if b == 1 and c == 1:
        for i in range(a):
            out.append(_sum(p, _scaled(ua, i)))
        return
    if a == 1:
        if b >= c:
            walk(p, B, C, A, out)
        else:
            walk(p, C, B, A, out)
        return
    kind, s = choose_cut(a, b, c)
    if kind == "W":
        a1 = s[0]
        walk(p, _scaled(ua, a1), B, C, out)
        walk(_sum(p, _scaled(ua, a1)), _scaled(ua, a - a1), B, C, out)
    elif kind in ("UB", "UC"):
        # the U in the plane of A and M (M = B or C), N is the untouched axis
        (m, um, N) = (b, ub, C) if kind == "UB" else (c, uc, B)
        a1, m1 = s
        # up along M through the near corner piece
        walk(p, _scaled(um, m1), _scaled(ua, a1), N, out)
        # across the whole major axis through the far strip
        walk(_sum(p, _scaled(um, m1)), A, _scaled(um, m - m1), N, out)
        # back down along M through the other corner piece, towards the start side of A
        walk(_sum(p, _scaled(ua, a - 1), _scaled(um, m1 - 1)), _scaled(um, -m1), _scaled(ua, -(a - a1)), N, out)
    else:
        a1, b1, c1 = s
        a2, b2, c2 = a - a1, b - b1, c - c1
        # near corner piece, up along B
        walk(p, _scaled(ub, b1), _scaled(uc, c1), _scaled(ua, a1), out)
        # near half of A, far part of B, all of C: out along C
        walk(_sum(p, _scaled(ub, b1)), C, _scaled(ua, a1), _scaled(ub, b2), out)
        # near part of B, far part of C: across the whole major axis
        walk(_sum(p, _scaled(ub, b1 - 1), _scaled(uc, c - 1)), A, _scaled(ub, -b1), _scaled(uc, -c2), out)
        # far half of A, far part of B, all of C: back along C
        walk(_sum(p, _scaled(ua, a - 1), _scaled(ub, b1), _scaled(uc, c - 1)), _scaled(uc, -c), _scaled(ub, b2),
             _scaled(ua, -a2), out)
        # far corner piece, down along B to the end of the major edge
        walk(_sum(p, _scaled(ua, a - 1), _scaled(ub, b1 - 1)), _scaled(ub, -b1), _scaled(ua, -a2), _scaled(uc, c1), out)


def box_curve(a: int, b: int, c: int) -> np.ndarray:
    """[a*b*c, 3] cells of an a x b x c box with axis 0 as the major axis."""
    limit = sys.getrecursionlimit()
    sys.setrecursionlimit(max(limit, 10000))
    try:
        out: List[Vec] = []
        walk((0, 0, 0), (a, 0, 0), (0, b, 0), (0, 0, c), out)
    finally:
        sys.setrecursionlimit(limit)
    return np.asarray(out, dtype=np.int64).reshape(-1, 3)


def axis_roles(grid: Sequence[int]) -> Tuple[int, int, int]:
    """(major, B, C) as indices into (T, Y, X)."""
    even = [i for i in range(3) if grid[i] % 2 == 0]
    pool = even if even else [0, 1, 2]
    major = max(pool, key=lambda i: (grid[i], -i))
    rest = [i for i in range(3) if i != major]
    second = max(rest, key=lambda i: (grid[i], -i))
    third = [i for i in rest if i != second][0]
    return major, second, third


def grid_curve(grid: Sequence[int]) -> np.ndarray:
    """[T*Y*X, 3] cells (t, y, x) in curve order."""
    major, second, third = axis_roles(grid)
    cells = box_curve(grid[major], grid[second], grid[third])
    out = np.empty_like(cells)
    out[:, major], out[:, second], out[:, third] = cells[:, 0], cells[:, 1], cells[:, 2]
    return out


def token_order(grid: Sequence[int], n_prefix: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """(order, inverse), both int32 [n_prefix + T*Y*X].

    The reordered sequence holds at position i the token that the raster-order sequence (t major,
    then y, then x, after n_prefix leading tokens that keep their places) holds at order[i];
    inverse[order[i]] = i.
    """
    T, Y, X = grid
    cells = grid_curve(grid)
    raster = (cells[:, 0] * Y + cells[:, 1]) * X + cells[:, 2]
    order = np.concatenate([np.arange(n_prefix, dtype=np.int64), n_prefix + raster]).astype(np.int32)
    inverse = np.empty_like(order)
    inverse[order] = np.arange(order.size, dtype=np.int32)
    return order, inverse


def permute_tokens(x: np.ndarray, order: np.ndarray) -> np.ndarray:
    """out[..., i, :] = x[..., order[i], :] for a [..., L, d] array."""
    return np.take(x, order, axis=-2)
