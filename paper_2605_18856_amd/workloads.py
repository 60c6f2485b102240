"""Seeded synthetic games and candidate sets (numpy only).

This module draws inputs; it holds none of the sweep's arithmetic and loads no
native code.  Both the GPU library's callers and the CPU checker take their
inputs from here so that they see the same bits.

The five games follow the benchmark configurations this repository is measured
on (shapes, value distributions, priors); every draw uses
``numpy.random.Generator(PCG64(seed))`` with the fixed seeds below.
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

PAYOFF_SEED = 1000
PRIOR_SEED = 2000
CANDIDATE_SEED = 3000


@dataclass
class Game:
    name: str
    m: int
    n: int
    K: int
    A: np.ndarray            # float32 [K][m][n]  leader payoffs
    B: np.ndarray            # float32 [K][m][n]  follower payoffs
    prior: np.ndarray        # float32 [K]
    storage: str = "f32"     # "f32" or "bf16": how the library is asked to store payoffs
    candidates: str = "dirichlet"   # "dirichlet" or "lattice"
    count: int = 0           # number of candidates of the full configuration
    lattice_N: Optional[int] = None
    chunk: Optional[int] = None     # candidates per sweep call when streamed
    candidate_seed: int = 0
    notes: dict = field(default_factory=dict)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    bias = ((bits >> np.uint64(16)) & np.uint64(1)) + np.uint64(0x7FFF)
    out = ((bits + bias) & np.uint64(0xFFFF0000)).astype(np.uint32)
    return out.view(np.float32).reshape(a.shape)


def _dirichlet_prior(rng, K, alpha):
    p = rng.dirichlet(np.full(K, alpha)).astype(np.float32)
    # keep the fp32 prior on the simplex to well within the library's 1e-6 check
    p64 = p.astype(np.float64)
    p = (p64 / p64.sum()).astype(np.float32)
    return p


def game(config: int, variant: str = "") -> Game:
    """config 1..5 (file order of the benchmark list).  variant "ties" (config 5
    only) duplicates follower-payoff columns so that exact follower ties occur."""
    rng = np.random.Generator(np.random.PCG64(PAYOFF_SEED + config))
    prng = np.random.Generator(np.random.PCG64(PRIOR_SEED + config))
    cseed = CANDIDATE_SEED + config
    if config == 1:
        m, n, K = 3, 3, 2
        A = rng.random((K, m, n)).astype(np.float32)       # fp64 draw, rounded once
        B = rng.random((K, m, n)).astype(np.float32)
        prior = np.array([0.7, 0.3], dtype=np.float32)
        return Game("tiny_m3n3K2_latticeN100", m, n, K, A, B, prior, "f32", "lattice",
                    5151, 100, None, cseed)
    if config == 2:
        m, n, K = 8, 8, 4
        A = rng.standard_normal((K, m, n)).astype(np.float32)
        B = rng.standard_normal((K, m, n)).astype(np.float32)
        prior = _dirichlet_prior(prng, K, 1.0)
        return Game("m8n8K4_dirichlet_2p20", m, n, K, A, B, prior, "f32", "dirichlet",
                    1 << 20, None, None, cseed)
    if config == 3:
        m, n, K = 32, 32, 16
        A = rng.standard_normal((K, m, n))
        rho = rng.uniform(-1.0, 1.0, size=K)
        Z = rng.standard_normal((K, m, n))
        B = rho[:, None, None] * A + np.sqrt(1.0 - rho ** 2)[:, None, None] * Z
        prior = _dirichlet_prior(prng, K, 0.5)
        return Game("misalign_m32n32K16_dirichlet_2p24", m, n, K, A.astype(np.float32),
                    B.astype(np.float32), prior, "f32", "dirichlet", 1 << 24, None, None,
                    cseed, {"rho": rho})
    if config == 4:
        m, n, K = 64, 128, 64
        A = round_to_bf16(rng.uniform(-1.0, 1.0, (K, m, n)).astype(np.float32))
        B = round_to_bf16(rng.uniform(-1.0, 1.0, (K, m, n)).astype(np.float32))
        prior = np.full(K, 1.0 / K, dtype=np.float32)
        return Game("dense_m64n128K64_bf16_2p26", m, n, K, A, B, prior, "bf16", "dirichlet",
                    1 << 26, None, 1 << 22, cseed)
    if config == 5:
        m, n, K = 128, 256, 256
        A = rng.integers(0, 8, (K, m, n)).astype(np.float32)
        B = rng.integers(0, 8, (K, m, n)).astype(np.float32)
        prior = _dirichlet_prior(prng, K, 1.0)
        name = "ties_m128n256K256_int_2p24"
        if variant == "ties":
            # every 8th follower column is copied onto its right neighbour; the leader
            # columns stay different, so the tie-break has something to decide
            for j in range(0, n - 1, 8):
                B[:, :, j + 1] = B[:, :, j]
            name += "_dupcols"
        return Game(name, m, n, K, A, B, prior, "f32", "dirichlet", 1 << 24, None, None, cseed)
    raise ValueError("config must be 1..5")


def small_game(m, n, K, seed, kind="normal", storage="f32") -> Game:
    """A random game of arbitrary shape for tests: kind in normal|uniform|int|dup."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if kind == "normal":
        A = rng.standard_normal((K, m, n)).astype(np.float32)
        B = rng.standard_normal((K, m, n)).astype(np.float32)
    elif kind == "uniform":
        A = rng.uniform(-1, 1, (K, m, n)).astype(np.float32)
        B = rng.uniform(-1, 1, (K, m, n)).astype(np.float32)
    elif kind in ("int", "dup"):
        A = rng.integers(0, 8, (K, m, n)).astype(np.float32)
        B = rng.integers(0, 8, (K, m, n)).astype(np.float32)
        if kind == "dup":
            for j in range(0, n - 1, 3):
                B[:, :, j + 1] = B[:, :, j]
    else:
        raise ValueError(kind)
    if storage == "bf16":
        A, B = round_to_bf16(A), round_to_bf16(B)
    prior = _dirichlet_prior(rng, K, 1.0)
    return Game(f"small_{kind}_m{m}n{n}K{K}_s{seed}", m, n, K, A, B, prior, storage,
                "dirichlet", 0, None, None, seed)


def host_candidates(m, count, seed, kind="dirichlet") -> np.ndarray:
    """Host-drawn float32 candidates [count][m] for tests: 'dirichlet' (numpy's own
    sampler), 'sparse' (few non-zeros), 'vertex' (unit vectors, cyclic), 'dyadic'
    (multiples of 1/16 summing to 1; exact in any binary format)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if kind == "dirichlet":
        return rng.dirichlet(np.ones(m), size=count).astype(np.float32)
    if kind == "sparse":
        X = np.zeros((count, m), dtype=np.float64)
        for c in range(count):
            nz = rng.choice(m, size=min(m, 1 + int(rng.integers(0, 3))), replace=False)
            X[c, nz] = rng.dirichlet(np.ones(len(nz)))
        return X.astype(np.float32)
    if kind == "vertex":
        X = np.zeros((count, m), dtype=np.float32)
        X[np.arange(count), np.arange(count) % m] = 1.0
        return X
    if kind == "dyadic":
        X = np.zeros((count, m), dtype=np.float32)
        for c in range(count):
            cuts = np.sort(rng.integers(0, 17, size=m - 1))
            parts = np.diff(np.concatenate([[0], cuts, [16]]))
            X[c] = parts / 16.0
        return X
    raise ValueError(kind)
