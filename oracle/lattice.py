"""Simplex lattice of resolution N in m parts, in exact integer arithmetic.

TEST INFRASTRUCTURE ONLY.  The lattice is the set of x = k/N with k a vector of m
non-negative integers summing to N (the compositions of N into m parts), listed in
ascending lexicographic order of (k_0, ..., k_{m-1}): rank 0 is (0, ..., 0, N) and the
last rank is (N, 0, ..., 0).  There are C(N+m-1, m-1) of them.

``unrank`` walks the definition: for component i it skips, one value of k_i at a time,
the block of compositions that start with that value (a block of the remaining total R'
into q parts has C(R'+q-1, q-1) members), until the rank falls inside a block.
A candidate is fl32(k_i) / fl32(N), one correctly rounded fp32 division per component.
"""
from math import comb

import numpy as np


def count(m: int, N: int) -> int:
    return comb(N + m - 1, m - 1)


def unrank(r: int, m: int, N: int):
    if not 0 <= r < count(m, N):
        raise ValueError("rank out of range")
    k = []
    rem = N
    for i in range(m - 1):
        q = m - 1 - i                      # parts left after this one
        v = 0
        while True:
            block = comb(rem - v + q - 1, q - 1)
            if r < block:
                break
            r -= block
            v += 1
        k.append(v)
        rem -= v
    k.append(rem)
    return k


def rank(k, N: int) -> int:
    m = len(k)
    r = 0
    rem = N
    for i in range(m - 1):
        q = m - 1 - i
        for v in range(k[i]):
            r += comb(rem - v + q - 1, q - 1)
        rem -= k[i]
    return r


def compositions(m: int, N: int) -> np.ndarray:
    """All compositions in lexicographic order, int64[count][m], by direct recursion
    (independent of unrank)."""
    out = []

    def rec(prefix, rem, parts):
        if parts == 1:
            out.append(prefix + [rem])
            return
        for v in range(rem + 1):
            rec(prefix + [v], rem - v, parts - 1)

    rec([], N, m)
    return np.asarray(out, dtype=np.int64).reshape(-1, m)


def points_f32(m: int, N: int, first: int = 0, cnt: int = None) -> np.ndarray:
    """Candidates float32[cnt][m] for ranks first..first+cnt-1: fl32(k)/fl32(N)."""
    total = count(m, N)
    if cnt is None:
        cnt = total - first
    k = np.asarray([unrank(r, m, N) for r in range(first, first + cnt)],
                   dtype=np.int64).reshape(-1, m)
    return (k.astype(np.float32) / np.float32(N)).astype(np.float32)


def points_around_f32(m: int, N: int, centre, radius, first: int = 0, cnt: int = None) -> np.ndarray:
    """The lattice shrunk towards `centre`: every point t of ``points_f32`` becomes
    (1 - radius) * centre + radius * t, each component as three separately rounded float32
    operations fl(fl(radius * t) + fl(fl(1 - radius) * centre))."""
    t = points_f32(m, N, first, cnt)
    r = np.float32(radius)
    omr = np.float32(np.float32(1.0) - r)
    c = np.asarray(centre, dtype=np.float32)
    return ((r * t).astype(np.float32) + (omr * c).astype(np.float32)[None, :]).astype(np.float32)
