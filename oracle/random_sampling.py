"""CPU oracle for seeded per-block random sampling -- TEST INFRASTRUCTURE ONLY.

Alg. 3 step 2 samples k tokens "randomly" from every block.  Here the draw is made reproducible
with a counter-based generator, Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel
random numbers: as easy as 1, 2, 3", SC'11), written from its published definition:

    round:   (hi0, lo0) = M0 * c0,  (hi1, lo1) = M1 * c2      (32 x 32 -> 64 bit products)
             c <- (hi1 ^ c1 ^ k0,  lo1,  hi0 ^ c3 ^ k1,  lo0)
             k <- (k0 + W0, k1 + W1)                           (after every round but the last)
    M0 = 0xD2511F53, M1 = 0xCD9E8D57, W0 = 0x9E3779B9, W1 = 0xBB67AE85

Reading (the paper gives no procedure): for block `blk` of slab `slab` (= batch * H + head) every
position j in [0, b) gets the 32-bit word r_j = Philox(counter = (j, blk, slab, 0),
key = (seed low word, seed high word))[0]; the k positions with the smallest (r_j, j) are the
sample, listed in ascending position.  Q and K use the same positions (one table per slab).

The importance map for a per-block table is Alg. 3 steps 3-5 written out in numpy fp64.
"""

from __future__ import annotations

import math
from typing import Optional, Sequence

import numpy as np

M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def philox4x32_10(counter: Sequence[int], key: Sequence[int]):
    c0, c1, c2, c3 = (int(x) & MASK for x in counter)
    k0, k1 = (int(x) & MASK for x in key)
    for r in range(10):
        p0 = M0 * c0
        p1 = M1 * c2
        hi0, lo0 = p0 >> 32, p0 & MASK
        hi1, lo1 = p1 >> 32, p1 & MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
        if r != 9:
            k0 = (k0 + W0) & MASK
            k1 = (k1 + W1) & MASK
    return c0, c1, c2, c3


def block_offsets(seed: int, slab: int, blk: int, b: int, k: int) -> np.ndarray:
    """The k sampled positions of one block, ascending."""
    key = (seed & MASK, (seed >> 32) & MASK)
    words = [(philox4x32_10((j, blk, slab, 0), key)[0], j) for j in range(b)]
    words.sort()
    return np.array(sorted(j for _, j in words[:k]), dtype=np.int64)


def offsets_table(seed: int, n_slabs: int, Nb: int, b: int, k: int) -> np.ndarray:
    """uint8 [n_slabs, Nb, k]."""
    t = np.zeros((n_slabs, Nb, k), np.uint8)
    for s in range(n_slabs):
        for i in range(Nb):
            t[s, i] = block_offsets(seed, s, i, b, k)
    return t


def p_imp_table(q: np.ndarray, k: np.ndarray, b: int, table: np.ndarray,
                scale: Optional[float] = None) -> np.ndarray:
    """Importance map of one slab [L, d] for a per-block table [Nb, ks] (Alg. 3 steps 3-5):
    soft-max over ALL valid sampled keys, maximum over the sampled pairs of each block pair.
    Samples that fall past L do not exist."""
    L, d = q.shape
    Nb, ks = table.shape
    scale = float(np.float32(1.0) / np.sqrt(np.float32(d))) if scale is None else scale
    pos = (np.arange(Nb)[:, None] * b + table.astype(np.int64)).reshape(-1)
    valid = pos < L
    blk = np.repeat(np.arange(Nb), ks)
    qs = q[pos[valid]].astype(np.float64)
    ks_ = k[pos[valid]].astype(np.float64)
    bq = blk[valid]
    s = scale * (qs @ ks_.T)
    s -= s.max(axis=1, keepdims=True)
    e = np.exp(s)
    p = e / e.sum(axis=1, keepdims=True)
    out = np.zeros((Nb, Nb))
    for i in range(Nb):
        ri = np.nonzero(bq == i)[0]
        if ri.size == 0:
            continue
        pi = p[ri]
        for j in range(Nb):
            cj = np.nonzero(bq == j)[0]
            if cj.size:
                out[i, j] = pi[:, cj].max()
    return out
