"""Seeded flat-Dirichlet candidate rows, in fp64.  TEST INFRASTRUCTURE ONLY.

A point uniform on the simplex (Dirichlet with all parameters 1) is a vector of m
independent unit exponentials divided by its sum (textbook construction).  The
uniforms come from a counter-based generator so that row c never depends on how the
rows are split over launches: Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw,
"Parallel random numbers: as easy as 1, 2, 3", SC'11), written here from that paper's
description:

    round:  (hi0, lo0) = M0 * c0,  (hi1, lo1) = M1 * c2      (32x32 -> 64 bit products)
            (c0, c1, c2, c3) <- (hi1 ^ c1 ^ k0,  lo1,  hi0 ^ c3 ^ k1,  lo0)
    between rounds the key is bumped: k0 += W0, k1 += W1     (mod 2^32)

Use here: key = (seed low word, seed high word); counter = (row low word, row high
word, b, 0) yields the four words for components 4b..4b+3 of that row.  A word w maps
to u = ((w >> 8) + 1) / 2^24, which lies in (0, 1], so ln u is finite; g = -ln u;
x_i = g_i / sum_i g_i (i ascending).  If every g is 0 the row is 1/m throughout.
"""
import numpy as np

M0 = np.uint64(0xD2511F53)
M1 = np.uint64(0xCD9E8D57)
W0 = 0x9E3779B9
W1 = 0xBB67AE85
MASK = np.uint64(0xFFFFFFFF)
SH = np.uint64(32)


def philox4x32_10(ctr, key):
    """ctr: uint32[..., 4], key: uint32[..., 2] (broadcastable) -> uint32[..., 4]."""
    ctr = np.asarray(ctr, dtype=np.uint32)
    key = np.asarray(key, dtype=np.uint32)
    c0, c1, c2, c3 = (ctr[..., q].astype(np.uint64) for q in range(4))
    k0 = key[..., 0].astype(np.uint64)
    k1 = key[..., 1].astype(np.uint64)
    for rnd in range(10):
        if rnd:
            k0 = (k0 + np.uint64(W0)) & MASK
            k1 = (k1 + np.uint64(W1)) & MASK
        p0 = M0 * c0
        p1 = M1 * c2
        hi0, lo0 = p0 >> SH, p0 & MASK
        hi1, lo1 = p1 >> SH, p1 & MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def word_to_uniform(w) -> np.ndarray:
    """A 32-bit generator word to u = ((w >> 8) + 1) / 2^24: the top 24 bits, shifted into (0, 1]."""
    w = np.asarray(w, dtype=np.uint32)
    return ((w >> np.uint32(8)).astype(np.float64) + 1.0) / 16777216.0


def uniforms(seed: int, first: int, count: int, m: int) -> np.ndarray:
    """u[count][m] in (0,1], float64 (each value is an integer multiple of 2^-24)."""
    rows = np.arange(first, first + count, dtype=np.uint64)
    nb = (m + 3) // 4
    ctr = np.zeros((count, nb, 4), dtype=np.uint32)
    ctr[:, :, 0] = (rows & MASK).astype(np.uint32)[:, None]
    ctr[:, :, 1] = (rows >> SH).astype(np.uint32)[:, None]
    ctr[:, :, 2] = np.arange(nb, dtype=np.uint32)[None, :]
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint32)
    w = philox4x32_10(ctr, key).reshape(count, nb * 4)[:, :m]
    return word_to_uniform(w)


def rows(seed: int, first: int, count: int, m: int) -> np.ndarray:
    """float64[count][m] flat-Dirichlet rows for global row indices first..first+count-1."""
    g = -np.log(uniforms(seed, first, count, m))
    s = np.zeros(count)
    for i in range(m):                     # ascending, as stated
        s = s + g[:, i]
    out = np.where(s[:, None] > 0, g / np.where(s > 0, s, 1.0)[:, None], 1.0 / m)
    return out


def rows_around(seed: int, first: int, count: int, m: int, centre, radius) -> np.ndarray:
    """``rows`` shrunk towards `centre`: (1 - radius) * centre + radius * row, in float64 (radius and
    1 - radius taken as the float32 numbers the library uses)."""
    r = np.float64(np.float32(radius))
    omr = np.float64(np.float32(np.float32(1.0) - np.float32(radius)))
    c = np.asarray(centre, dtype=np.float32).astype(np.float64)
    return r * rows(seed, first, count, m) + omr * c[None, :]
