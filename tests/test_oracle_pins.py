"""Pins for the CPU oracle (no GPU).  Each test checks the oracle against something the
mathematics fixes independently of the oracle's own loops: an exact LP solve, a closed
form, a hand-solved game, an exact-rational enumeration over follower profiles, or an
invariance."""
import os
from fractions import Fraction
from itertools import product

import numpy as np
import pytest

from oracle import lattice, sse_lp, sweep as osweep
from paper_2605_18856_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def lattice_points64(m, N):
    """Exact-in-fp64 lattice points k/N from the independent recursive enumeration."""
    return lattice.compositions(m, N).astype(np.float64) / float(N)


# ----------------------------------------------------------------------------- hand game
def _read_hand_2x2():
    rows = []
    for line in open(os.path.join(GOLDEN, "hand_tiebreak_2x2.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append([int(t) for t in line.split()])
    return rows


@pytest.mark.parametrize("N,num,den,k0,br", _read_hand_2x2())
def test_hand_2x2_tiebreak_is_load_bearing(N, num, den, k0, br):
    A = np.array([[[2, 4], [1, 3]]], dtype=np.float64)
    B = np.array([[[1, 0], [0, 1]]], dtype=np.float64)
    X = lattice_points64(2, N)
    r = osweep.sweep(A, B, [1.0], X)
    assert r.best_value == pytest.approx(num / den, abs=1e-15)
    assert X[r.best_index, 0] * N == pytest.approx(k0, abs=1e-12)
    assert r.best_br[0] == br


def _read_tie_cases():
    lines = [l.strip() for l in open(os.path.join(GOLDEN, "hand_tie_cases.txt"))]
    lines = [l for l in lines if l and not l.startswith("#")]
    cases, i = [], 0
    while i < len(lines):
        assert lines[i].startswith("case ")
        name = lines[i][5:]
        m, n = (int(t) for t in lines[i + 1].split())
        x = [float(t) for t in lines[i + 2].split()]
        Bm = [[float(t) for t in lines[i + 3 + r].split()] for r in range(m)]
        Am = [[float(t) for t in lines[i + 3 + m + r].split()] for r in range(m)]
        br, val = lines[i + 3 + 2 * m].split()
        cases.append(pytest.param(x, Bm, Am, int(br), float(val), id=name))
        i += 4 + 2 * m
    return cases


@pytest.mark.parametrize("x,Bm,Am,br,val", _read_tie_cases())
def test_hand_tie_cases(x, Bm, Am, br, val):
    r = osweep.sweep(np.array([Am]), np.array([Bm]), [1.0], np.array([x]))
    assert r.br[0, 0] == br
    assert r.values[0] == val


# ------------------------------------------------------- exact LP (multiple-LPs) solves
TINY_SHAPES = [(3, 3, 2), (2, 2, 3), (4, 2, 2), (3, 4, 1), (2, 3, 2)]


@pytest.mark.parametrize("shape", TINY_SHAPES)
@pytest.mark.parametrize("seed", [11, 12, 13])
def test_lattice_value_never_exceeds_lp_and_converges(shape, seed):
    m, n, K = shape
    g = workloads.small_game(m, n, K, seed, kind="uniform")
    v_lp, x_lp, prof = sse_lp.solve(g.A, g.B, g.prior)
    # the LP optimum is attained by its own profile at its own x
    v_prof, _ = osweep.value_under_profile(g.A, g.prior, x_lp, prof)
    assert v_prof == pytest.approx(v_lp, abs=1e-9)
    A64, B64, p64 = (a.astype(np.float64) for a in (g.A, g.B, g.prior))
    prev = -np.inf
    Ns = [4, 8, 16, 32, 64] if m <= 3 else [4, 8, 16, 32]
    for N in Ns:
        X = lattice_points64(m, N)
        r = osweep.sweep(g.A, g.B, g.prior, X)
        assert r.best_value <= v_lp + 1e-9            # V(x) <= V_LP for every x
        assert r.best_value >= prev - 1e-12           # N | N' => lattice_N inside lattice_N'
        prev = r.best_value
        # wherever the LP-optimal profile is a strict best response (checked with numpy,
        # not with the oracle), V(x) equals that profile's objective there
        slack = np.full(X.shape[0], np.inf)
        obj = np.zeros(X.shape[0])
        for t, j in enumerate(prof):
            U = X @ B64[t]
            others = np.delete(U, j, axis=1)
            slack = np.minimum(slack, U[:, j] - others.max(axis=1))
            obj += p64[t] * (X @ A64[t][:, j])
        inside = slack > 1e-9
        assert np.allclose(r.values[inside], obj[inside], atol=1e-12)
        assert np.all(r.br[inside] == np.array(prof))
        if inside.any():
            # convergence from below: a lattice point inside the optimal region within
            # distance d of the LP optimiser loses at most (max |A|) * d  (|A| <= 1 here)
            d = np.abs(X[inside] - x_lp).sum(axis=1).min()
            assert v_lp - r.best_value <= d + 1e-9


def test_config1_lattice_against_nine_lps():
    g = workloads.game(1)
    v_lp, x_lp, prof = sse_lp.solve(g.A, g.B, g.prior)
    X = lattice.points_f32(3, 100)
    assert X.shape == (5151, 3)
    r = osweep.sweep(g.A, g.B, g.prior, X)
    assert r.best_value <= v_lp + 1e-6
    assert v_lp - r.best_value <= 12.0 / 100
    # the sweep's winner plays into a profile the LP also rates at least as high as any
    # lattice point can reach
    assert np.all(r.values <= v_lp + 1e-6)
    # chain 5 | 10 | 20 | 40 | 80 | 160
    prev = -np.inf
    for N in (5, 10, 20, 40, 80, 160):
        rn = osweep.sweep(g.A, g.B, g.prior, lattice_points64(3, N), per_candidate=False)
        assert prev - 1e-12 <= rn.best_value <= v_lp + 1e-9
        prev = rn.best_value
    assert v_lp - prev <= 12.0 / 160


def test_perturbed_lp_optimum_reaches_lp_value():
    """Move the LP optimiser slightly into the interior of its profile's region: there the
    profile is the strict best response, so the oracle must return that profile and a
    value within O(eps) of V_LP."""
    from scipy.optimize import linprog
    hits = 0
    for seed in range(20, 30):
        g = workloads.small_game(3, 3, 2, seed, kind="uniform")
        A, B, p = g.A.astype(np.float64), g.B.astype(np.float64), g.prior.astype(np.float64)
        v_lp, x_lp, prof = sse_lp.solve(A, B, p)
        # centre of the profile's region: maximise the smallest best-response slack
        rows = []
        for t, j in enumerate(prof):
            for jp in range(3):
                if jp != j:
                    rows.append(np.concatenate([B[t][:, jp] - B[t][:, j], [1.0]]))
        res = linprog(np.array([0, 0, 0, -1.0]), A_ub=np.array(rows), b_ub=np.zeros(len(rows)),
                      A_eq=np.array([[1, 1, 1, 0.0]]), b_eq=[1.0],
                      bounds=[(0, None)] * 3 + [(None, 1.0)], method="highs")
        if res.status != 0 or res.x[3] < 1e-6:
            continue          # region has empty interior; nothing to test for this seed
        eps = 1e-6
        x = (1 - eps) * x_lp + eps * res.x[:3]
        r = osweep.sweep(A, B, p, x[None, :])
        assert tuple(r.br[0]) == prof
        assert abs(r.values[0] - v_lp) <= 1e-4
        hits += 1
    assert hits >= 5


# ------------------------------------------------------------ zero-sum closed forms
def test_zero_sum_single_type_is_maximin():
    rng = np.random.default_rng(5)
    for _ in range(5):
        M = rng.uniform(-1, 1, (3, 4))
        v_mm, _ = sse_lp.maximin(M)
        for N in (10, 40):
            X = lattice_points64(3, N)
            r = osweep.sweep(M[None], -M[None], [1.0], X)
            # independent formula: the follower minimises the leader's payoff
            direct = (X @ M).min(axis=1)
            assert np.allclose(r.values, direct, atol=1e-14)
            assert r.best_value == pytest.approx(direct.max(), abs=1e-14)
            assert r.best_value <= v_mm + 1e-9
        assert v_mm - r.best_value <= 8.0 / 40


def test_zero_sum_2x2_closed_form():
    # no saddle point: value (ad - bc)/(a + d - b - c) at x0 = (d - c)/(a + d - b - c)
    a, b, c, d = 3.0, -1.0, -2.0, 2.0
    M = np.array([[a, b], [c, d]])
    val = (a * d - b * c) / (a + d - b - c)          # 4/8 = 0.5
    x0 = (d - c) / (a + d - b - c)                   # 4/8 = 0.5
    X = lattice_points64(2, 8)
    r = osweep.sweep(M[None], -M[None], [1.0], X)
    assert r.best_value == val
    assert X[r.best_index, 0] == x0
    # matching pennies: value 0 at (1/2, 1/2)
    P = np.array([[1.0, -1.0], [-1.0, 1.0]])
    r = osweep.sweep(P[None], -P[None], [1.0], lattice_points64(2, 10))
    assert r.best_value == 0.0 and r.best_index == 5


# ------------------------------------------------------------ dominated strategies
def test_dominant_follower_column_gives_vertex_optimum():
    rng = np.random.default_rng(9)
    K, m, n, j0 = 3, 4, 5, 2
    A = rng.uniform(0, 1, (K, m, n))
    B = rng.uniform(0, 1, (K, m, n))
    B[:, :, j0] = B.max(axis=2) + 0.5                # column j0 strictly dominates, every type
    p = np.array([0.2, 0.5, 0.3])
    for N in (1, 3, 7):
        X = lattice_points64(m, N)
        r = osweep.sweep(A, B, p, X)
        assert np.all(r.br == j0)
        lin = X @ np.einsum("t,ti->i", p, A[:, :, j0])        # V is linear in x
        assert np.allclose(r.values, lin, atol=1e-14)
        istar = int(np.argmax(np.einsum("t,ti->i", p, A[:, :, j0])))
        assert X[r.best_index, istar] == 1.0
        assert np.all(r.best_br == j0)


# ------------------------------------------------- exact-rational profile enumeration
def _profile_enumeration_value(A, B, p, x):
    """V(x) as 'best objective over follower profiles that are best responses at x',
    in exact rational arithmetic (a different statement of the same number)."""
    K, m, n = A.shape
    F = lambda a: Fraction(a).limit_denominator(1 << 20)
    xq = [F(float(v)) for v in x]
    u = [[sum(xq[i] * F(float(B[t, i, j])) for i in range(m)) for j in range(n)] for t in range(K)]
    l = [[sum(xq[i] * F(float(A[t, i, j])) for i in range(m)) for j in range(n)] for t in range(K)]
    best = None
    for prof in product(range(n), repeat=K):
        if all(u[t][prof[t]] >= max(u[t]) for t in range(K)):
            val = sum(F(float(p[t])) * l[t][prof[t]] for t in range(K))
            if best is None or val > best:
                best = val
    return best, u, l


@pytest.mark.parametrize("kind", ["int", "dup"])
def test_against_exact_rational_profile_enumeration(kind):
    for seed in range(40, 46):
        g = workloads.small_game(3, 4, 2, seed, kind=kind)
        p = np.array([0.25, 0.75])
        X = workloads.host_candidates(3, 24, seed, "dyadic").astype(np.float64)
        r = osweep.sweep(g.A, g.B, p, X, diagnostics=True)
        for c in range(X.shape[0]):
            v, u, l = _profile_enumeration_value(g.A, g.B, p, X[c])
            assert Fraction(r.values[c]) == v
            for t in range(2):
                j = int(r.br[c, t])
                assert u[t][j] == max(u[t])                               # a best response
                tie = [q for q in range(4) if u[t][q] == u[t][j]]
                assert l[t][j] == max(l[t][q] for q in tie)               # leader-favourable
                assert j == min(q for q in tie if l[t][q] == l[t][j])     # then lowest index
        if kind == "dup":
            assert (r.gap == 0).any()      # the duplicated columns really produce ties


# ------------------------------------------------------------------------ invariances
def test_invariances():
    g = workloads.small_game(4, 5, 3, 77, kind="int")
    X = workloads.host_candidates(4, 200, 78, "dyadic").astype(np.float64)
    A, B, p = g.A.astype(np.float64), g.B.astype(np.float64), np.array([0.5, 0.25, 0.25])
    base = osweep.sweep(A, B, p, X, diagnostics=True)
    # positive-affine rescaling of each type's follower payoffs (exact: powers of two)
    B2 = B * np.array([2.0, 0.5, 4.0])[:, None, None] + np.array([1.0, -3.0, 8.0])[:, None, None]
    r = osweep.sweep(A, B2, p, X)
    assert np.array_equal(r.br, base.br) and np.array_equal(r.values, base.values)
    # affine map of leader payoffs maps values affinely (rows of X sum to 1 exactly)
    r = osweep.sweep(4.0 * A - 2.0, B, p, X)
    assert np.array_equal(r.br, base.br)
    assert np.allclose(r.values, 4.0 * base.values - 2.0, atol=1e-12)
    assert r.best_index == base.best_index
    # relabelling follower actions permutes the value-irrelevant labels only
    perm = np.array([3, 0, 4, 1, 2])
    r = osweep.sweep(A[:, :, perm], B[:, :, perm], p, X)
    assert np.array_equal(r.values, base.values)
    untied = base.gap > 0
    assert np.array_equal(perm[r.br][untied], base.br[untied])
    # point-mass prior is the single-type game
    r1 = osweep.sweep(A, B, np.array([0.0, 1.0, 0.0]), X)
    r2 = osweep.sweep(A[1:2], B[1:2], [1.0], X)
    assert np.array_equal(r1.values, r2.values) and np.array_equal(r1.br[:, 1], r2.br[:, 0])
    # duplicating candidates never moves the winner; ties go to the lowest index
    r = osweep.sweep(A, B, p, np.concatenate([X, X]))
    assert r.best_index == base.best_index and r.best_value == base.best_value
    # transposing the roles of leader and follower actions is NOT an invariance: a
    # non-square game would not even type-check, and on a square one the values move
    gs = workloads.small_game(4, 4, 1, 5, kind="int")
    Xs = workloads.host_candidates(4, 50, 6, "dyadic").astype(np.float64)
    ra = osweep.sweep(gs.A, gs.B, [1.0], Xs)
    rb = osweep.sweep(gs.A.transpose(0, 2, 1), gs.B.transpose(0, 2, 1), [1.0], Xs)
    assert not np.array_equal(ra.values, rb.values)


def test_threads_and_f32_input_do_not_change_results():
    g = workloads.game(2)
    X = workloads.host_candidates(8, 3000, 1, "dirichlet")
    a = osweep.sweep(g.A, g.B, g.prior, X, diagnostics=True, nthreads=1)
    b = osweep.sweep(g.A, g.B, g.prior, X.astype(np.float64), diagnostics=True, nthreads=4)
    assert np.array_equal(a.values, b.values) and np.array_equal(a.br, b.br)
    assert np.array_equal(a.gap, b.gap) and np.array_equal(a.scale, b.scale)
    assert (a.best_index, a.best_value) == (b.best_index, b.best_value)
    assert b.threads == 4
    # values and diagnostics against numpy's matmul (library routine) on the same data
    U = np.einsum("ci,tij->ctj", X.astype(np.float64), g.B.astype(np.float64))
    assert np.array_equal(U.argmax(axis=2), a.br)      # no exact ties for continuous draws
    Us = np.sort(U, axis=2)
    assert np.allclose(a.gap, Us[:, :, -1] - Us[:, :, -2], atol=1e-12)
    L = np.einsum("ci,tij->ctj", X.astype(np.float64), g.A.astype(np.float64))
    V = (np.take_along_axis(L, a.br[:, :, None], axis=2)[:, :, 0] * g.prior.astype(np.float64)).sum(1)
    assert np.allclose(a.values, V, atol=1e-12)
    assert a.best_index == int(np.argmax(V))


def test_empty_and_single_candidate():
    g = workloads.game(1)
    r = osweep.sweep(g.A, g.B, g.prior, np.zeros((0, 3)))
    assert r.best_index == -1
    r = osweep.sweep(g.A, g.B, g.prior, np.array([[1.0, 0.0, 0.0]]))
    assert r.best_index == 0


# ------------------------------------------------------ diagnostics: gap, scale, abs-scale
def test_scale_and_gap_on_a_hand_case_with_cancellation():
    """x = (1/2, 1/2); follower payoffs by hand: u = (1, 3/2, 0).  Top two actions are 1 and 0.
    Their sums of absolute terms are |-1| + |5/2| = 7/2 and 2 + 1 = 3, so scale = 7/2 and
    gap = 1/2.  Action 2 has the largest absolute sum (100) but is not among the top two, and
    every action's terms cancel in part, so |sum| and sum|.| differ: a scale taken over all
    actions (100), of the maximiser alone, or as |u| (3/2) fails here."""
    B = np.array([[[4.0, -2.0, 100.0], [-2.0, 5.0, -100.0]]])
    A = np.array([[[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]]])
    r = osweep.sweep(A, B, [1.0], np.array([[0.5, 0.5]]), diagnostics=True)
    assert r.br[0, 0] == 1
    assert r.gap[0, 0] == 0.5
    assert r.scale[0, 0] == 3.5
    # runner-up with the larger absolute sum: swap the roles (u = (3/2, 1, 0); sums 3, 7/2)
    B2 = np.array([[[5.0, -1.0, 100.0], [-2.0, 3.0, -100.0]]])
    r2 = osweep.sweep(A, B2, [1.0], np.array([[0.5, 0.5]]), diagnostics=True)
    assert r2.br[0, 0] == 0 and r2.gap[0, 0] == 0.5 and r2.scale[0, 0] == 3.5
    # one action only: no runner-up
    r1 = osweep.sweep(A[:, :, :1], B[:, :, :1], [1.0], np.array([[0.5, 0.5]]), diagnostics=True)
    assert np.isinf(r1.gap[0, 0]) and r1.scale[0, 0] == 3.0


def test_scale_on_a_generic_game_against_numpy():
    g = workloads.small_game(7, 6, 3, 41, kind="normal")
    X = workloads.host_candidates(7, 500, 42, "dirichlet").astype(np.float64)
    r = osweep.sweep(g.A, g.B, g.prior, X, diagnostics=True)
    B64 = g.B.astype(np.float64)
    U = np.einsum("ci,tij->ctj", X, B64)
    S = np.einsum("ci,tij->ctj", np.abs(X), np.abs(B64))           # sum_i |x_i B_t[i][j]| (x >= 0 or not)
    order = np.argsort(-U, axis=2, kind="stable")
    top2 = np.take_along_axis(S, order[:, :, :2], axis=2)
    assert np.allclose(r.scale, top2.max(axis=2), rtol=1e-13, atol=0)
    assert np.allclose(r.gap, np.take_along_axis(U, order[:, :, :1], 2)[:, :, 0]
                       - np.take_along_axis(U, order[:, :, 1:2], 2)[:, :, 0], atol=1e-13)
    # candidates with negative components: absolute values are taken of the products
    Xn = X.copy()
    Xn[:, ::2] *= -1.0
    rn = osweep.sweep(g.A, g.B, g.prior, Xn, diagnostics=True)
    Un = np.einsum("ci,tij->ctj", Xn, B64)
    on = np.argsort(-Un, axis=2, kind="stable")
    assert np.allclose(rn.scale, np.take_along_axis(S, on[:, :, :2], axis=2).max(axis=2), rtol=1e-13)


def test_value_under_profile_and_its_abs_scale():
    """Hand case: p = (1/4, 3/4), x = (1/2, 1/2); type 0 told to play the column (2, -2):
    l = 0, sum|.| = 2; type 1 the column (-4, 1): l = -3/2, sum|.| = 5/2.
    V = -9/8, abs-scale = 1/2 + 15/8 = 19/8 (not |V|, and not unweighted)."""
    A = np.array([[[9.0, 2.0], [9.0, -2.0]], [[-4.0, 7.0], [1.0, 7.0]]])
    v, s = osweep.value_under_profile(A, [0.25, 0.75], [0.5, 0.5], [1, 0])
    assert v == -1.125 and s == 2.375
    # generic data against numpy
    g = workloads.small_game(9, 5, 4, 43, kind="normal")
    rng = np.random.Generator(np.random.PCG64(44))
    for _ in range(20):
        x = rng.standard_normal(9)
        br = rng.integers(0, 5, 4)
        v, s = osweep.value_under_profile(g.A, g.prior, x, br)
        cols = np.stack([g.A[t, :, br[t]].astype(np.float64) for t in range(4)])       # [K][m]
        p = g.prior.astype(np.float64)
        assert v == pytest.approx(float(p @ (cols @ x)), rel=1e-13, abs=1e-15)
        assert s == pytest.approx(float(p @ (np.abs(cols) @ np.abs(x))), rel=1e-13)


# --------------------------------------------------------- operand rounding fed to the oracle
def test_round_to_bf16_matches_an_independent_conversion():
    """The bf16 operands the oracle is fed come from workloads.round_to_bf16; PyTorch's CPU
    float32 -> bfloat16 conversion (round to nearest, ties to even) is the independent routine."""
    import torch
    rng = np.random.Generator(np.random.PCG64(45))
    vals = [rng.standard_normal(1 << 18).astype(np.float32),
            (rng.standard_normal(1 << 16) * 1e-30).astype(np.float32),
            (rng.standard_normal(1 << 16) * 1e30).astype(np.float32)]
    # every finite upper half with the lower half at, just below and just above the halfway point,
    # and at the extremes: ties go to the even upper half, everything else to the nearest
    hi = np.arange(1 << 16, dtype=np.uint32) << np.uint32(16)
    for lo in (0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF):
        vals.append((hi | np.uint32(lo)).view(np.float32))
    x = np.concatenate(vals)
    x = x[np.isfinite(x)]
    ours = workloads.round_to_bf16(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    fin = np.isfinite(ref)                       # values that round up to infinity: compare bits too
    assert np.array_equal(ours.view(np.uint32), ref.view(np.uint32))
    assert fin.sum() > 0.99 * x.size
    assert np.array_equal(workloads.round_to_bf16(ours), ours)                # idempotent
    assert (ours.view(np.uint32) & np.uint32(0xFFFF) == 0).all()
