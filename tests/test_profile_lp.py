"""The profile linear program (bsse_profile_lp, host code of the library; needs no GPU): against
closed forms of a hand-solved game, against scipy's HiGHS through the oracle's LP module on
random and degenerate games, and against the full multiple-LPs solve."""
from itertools import product

import numpy as np
import pytest

from oracle import sse_lp
from oracle import sweep as osweep
from paper_2605_18856_amd import bsse, workloads


def _feasible_point_ok(A, B, prior, profile, x, value, tol=1e-8):
    A = np.asarray(A, np.float64); B = np.asarray(B, np.float64); p = np.asarray(prior, np.float64)
    assert abs(x.sum() - 1.0) <= 1e-12 and (x >= 0).all()
    obj = sum(p[t] * x @ A[t][:, j] for t, j in enumerate(profile))
    assert abs(obj - value) <= tol * max(1.0, abs(value))
    for t, j in enumerate(profile):
        u = x @ B[t]
        assert (u[j] >= u - tol * max(1.0, np.abs(u).max())).all()


def test_hand_2x2_closed_forms():
    """A = [[2,4],[1,3]], B = [[1,0],[0,1]] (tests/golden/hand_tiebreak_2x2.txt): column 1 is a best
    response for x0 <= 1/2, where the leader gets 3 + x0: optimum 3.5 at (1/2, 1/2); column 0 for
    x0 >= 1/2 with 1 + x0: optimum 2 at (1, 0)."""
    A = np.array([[[2, 4], [1, 3]]], np.float32)
    B = np.array([[[1, 0], [0, 1]]], np.float32)
    ok, v, x = bsse.bsse_profile_lp(A, B, [1.0], [1])
    assert ok and abs(v - 3.5) < 1e-12 and np.allclose(x, [0.5, 0.5], atol=1e-12)
    ok, v, x = bsse.bsse_profile_lp(A, B, [1.0], [0])
    assert ok and abs(v - 2.0) < 1e-12 and np.allclose(x, [1.0, 0.0], atol=1e-12)
    # the oracle's single-profile routine is held to the same closed forms
    ok, v, x = sse_lp.profile_lp(A, B, [1.0], [1])
    assert ok and abs(v - 3.5) < 1e-9 and np.allclose(x, [0.5, 0.5], atol=1e-9)
    ok, v, x = sse_lp.profile_lp(A, B, [1.0], [0])
    assert ok and abs(v - 2.0) < 1e-9 and np.allclose(x, [1.0, 0.0], atol=1e-9)


def test_strictly_dominated_action_is_infeasible():
    B = np.array([[[3, 1, 0], [2, 1, 1], [5, 4, 2]]], np.float32)      # column 0 beats 1 and 2 in every row
    A = np.array([[[1, 2, 3], [4, 5, 6], [7, 8, 9]]], np.float32)
    assert bsse.bsse_profile_lp(A, B, [1.0], [1])[0] is False
    assert bsse.bsse_profile_lp(A, B, [1.0], [2])[0] is False
    assert sse_lp.profile_lp(A, B, [1.0], [1])[0] is False
    assert sse_lp.profile_lp(A, B, [1.0], [2])[0] is False
    ok, v, x = bsse.bsse_profile_lp(A, B, [1.0], [0])
    assert ok and abs(v - 7.0) < 1e-12 and np.allclose(x, [0, 0, 1], atol=1e-12)   # free choice of row


@pytest.mark.parametrize("shape,seed", [((3, 3, 2), 1), ((4, 3, 2), 2), ((5, 4, 2), 3), ((3, 2, 4), 4),
                                        ((6, 5, 1), 5), ((2, 6, 2), 6)])
def test_every_profile_against_highs(shape, seed):
    m, n, K = shape
    game = workloads.small_game(m, n, K, seed=seed, kind="normal")
    best = -np.inf
    n_feasible = 0
    for prof in product(range(n), repeat=K):
        ok, v, x = bsse.bsse_profile_lp(game.A, game.B, game.prior, prof)
        ok_ref, v_ref, _ = sse_lp.profile_lp(game.A, game.B, game.prior, prof)
        assert ok == ok_ref, prof
        if ok:
            assert abs(v - v_ref) <= 1e-8 * max(1.0, abs(v_ref)), prof
            _feasible_point_ok(game.A, game.B, game.prior, prof, x, v)
            best = max(best, v)
            n_feasible += 1
    assert n_feasible >= 1
    v_sse, _, _ = sse_lp.solve(game.A, game.B, game.prior)
    assert abs(best - v_sse) <= 1e-8 * max(1.0, abs(v_sse))


@pytest.mark.parametrize("kind", ["int", "dup"])
def test_degenerate_games_against_highs(kind):
    """Small-integer payoffs and duplicated follower columns: many constraints are active at once
    (degenerate vertices), and duplicated columns make a region's constraints linearly dependent."""
    game = workloads.small_game(5, 6, 2, seed=9, kind=kind)
    for prof in product(range(6), repeat=2):
        ok, v, x = bsse.bsse_profile_lp(game.A, game.B, game.prior, prof)
        ok_ref, v_ref, _ = sse_lp.profile_lp(game.A, game.B, game.prior, prof)
        assert ok == ok_ref, prof
        if ok:
            assert abs(v - v_ref) <= 1e-8 * max(1.0, abs(v_ref)), prof
            _feasible_point_ok(game.A, game.B, game.prior, prof, x, v)


@pytest.mark.parametrize("shape", [(16, 16, 8), (32, 32, 16), (64, 128, 8)])
def test_realised_profiles_of_larger_games(shape):
    """Profiles that are best responses at some x (taken from the oracle's sweep, so feasible by
    construction): K(n-1) up to 1016 constraints, m up to 64 rows in the dual tableau."""
    m, n, K = shape
    game = workloads.small_game(m, n, K, seed=m + K, kind="normal")
    X = workloads.host_candidates(m, 3, seed=4, kind="dirichlet")
    ref = osweep.sweep(game.A, game.B, game.prior, X, nthreads=4)
    for c in range(3):
        prof = ref.br[c]
        ok, v, x = bsse.bsse_profile_lp(game.A, game.B, game.prior, prof)
        ok_ref, v_ref, _ = sse_lp.profile_lp(game.A, game.B, game.prior, prof)
        assert ok and ok_ref
        assert abs(v - v_ref) <= 1e-7 * max(1.0, abs(v_ref))
        assert v >= ref.values[c] - 1e-9                # the candidate itself is feasible for it
        _feasible_point_ok(game.A, game.B, game.prior, prof, x, v, tol=1e-7)


def test_argument_errors():
    A = np.zeros((1, 2, 2), np.float32)
    with pytest.raises(bsse.BsseError) as e:
        bsse.bsse_profile_lp(A, A, [1.0], [2])
    assert e.value.status == bsse.BSSE_EINVAL
    bad = A.copy(); bad[0, 0, 0] = np.inf
    with pytest.raises(bsse.BsseError) as e:
        bsse.bsse_profile_lp(bad, A, [1.0], [0])
    assert e.value.status == bsse.BSSE_ENOTFINITE
    L = bsse.lib()
    assert L.bsse_polish(None, None, None, None, None, None) == bsse.BSSE_EINVAL
