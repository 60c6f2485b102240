"""LP polish of a sweep result (bsse_polish) against the exact multiple-LPs solve of the oracle's
LP module and hand-solved cases."""
import numpy as np
import pytest

from oracle import sse_lp
from oracle import sweep as osweep
from paper_2605_18856_amd import bsse, workloads
from tests import parity
from tests.test_gpu_parity import _make

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def test_hand_2x2_odd_lattice_is_polished_to_the_tie_point():
    """Odd N misses x = (1/2, 1/2): the lattice optimum is 3 + floor(N/2)/N with best response 1
    (tests/golden/hand_tiebreak_2x2.txt).  The program of profile (1) has its vertex exactly at
    (1/2, 1/2), where the follower is indifferent and the leader-favourable rule keeps column 1."""
    A = np.array([[[2, 4], [1, 3]]], np.float32)
    B = np.array([[[1, 0], [0, 1]]], np.float32)
    with bsse.bsse_create(2, 2, 1, A, B, np.ones(1, np.float32)) as g:
        for N in (1, 3, 5, 7, 101):
            bsse.bsse_lattice(g, N)
            out = bsse.bsse_sweep(g)
            assert abs(out.best_value - (3 + (N // 2) / N)) < 1e-6
            pol = bsse.bsse_polish(g)
            assert pol.point == 0 and np.array_equal(pol.x, np.float32([0.5, 0.5]))
            assert pol.value == 3.5 and pol.lp_value == pytest.approx(3.5, abs=1e-12)
            assert pol.best_response[0] == 1
            # the other profile's region is x0 >= 1/2 with optimum 2 at (1, 0)
            other = bsse.bsse_polish(g, profile=[0])
            assert other.lp_value == pytest.approx(2.0, abs=1e-12)
            assert other.value >= out.best_value          # never worse than the sweep's winner


def test_config1_polish_reaches_the_equilibrium_value():
    game = workloads.game(1)
    v_sse, x_sse, prof_sse = sse_lp.solve(game.A, game.B, game.prior)
    with _make(game) as g:
        for N in (10, 25, 100):
            bsse.bsse_lattice(g, N)
            out = bsse.bsse_sweep(g)
            pol = bsse.bsse_polish(g)
            assert out.best_value - 1e-6 <= pol.value <= v_sse + 1e-5
            assert pol.lp_value <= v_sse + 1e-9
            if tuple(out.best_response) == tuple(prof_sse):
                assert pol.lp_value == pytest.approx(v_sse, abs=1e-8)
                assert pol.value >= v_sse - 2e-5 * max(1.0, abs(v_sse))
            # the polished point really has the reported value (oracle, under the reported profile)
            v_ref, sc = osweep.value_under_profile(game.A, game.prior, pol.x.astype(np.float64),
                                                   pol.best_response)
            assert abs(pol.value - v_ref) <= 1e-5 * max(sc, 1e-30)


@pytest.mark.parametrize("shape,storage", [((8, 8, 4), "f32"), ((5, 7, 3), "f32"), ((16, 16, 4), "f32"),
                                           ((32, 32, 4), "f32"), ((64, 128, 2), "bf16")])
def test_polish_improves_a_coarse_sweep(shape, storage):
    """A few hundred random candidates leave room: the polished value must be at least the sweep's,
    at most the profile's program optimum (+ rounding), and consistent with the oracle at x_out."""
    torch = _torch()
    m, n, K = shape
    game = workloads.small_game(m, n, K, seed=100 + m, kind="uniform" if storage == "bf16" else "normal",
                                storage=storage)
    tol = parity.TOL_BF16 if storage == "bf16" else parity.TOL_F32
    X = workloads.host_candidates(m, 400, seed=12, kind="dirichlet")
    with _make(game) as g:
        Xd = torch.from_numpy(X).cuda()
        out = bsse.bsse_sweep(g, Xd, 400)
        pol = bsse.bsse_polish(g)
        again = bsse.bsse_sweep(g, Xd, 400)               # the handle still sweeps as before
    assert again.best_index == out.best_index and again.best_value == out.best_value
    assert pol.value >= out.best_value
    ok, v_lp, x_lp = sse_lp.profile_lp(game.A, game.B, game.prior, out.best_response)
    assert ok and pol.lp_value == pytest.approx(v_lp, rel=1e-7, abs=1e-7)
    A, B, xo = parity.oracle_inputs(game, pol.x[None, :])
    v_ref, sc = osweep.value_under_profile(A, game.prior, xo[0].astype(np.float64), pol.best_response)
    assert abs(pol.value - v_ref) <= tol * max(sc, 1e-30)
    # under bf16 storage the kernels see rounded operands, the program the unrounded ones: only
    # the fp32 path is held to the program's optimum as an upper bound
    if storage == "f32" and tuple(pol.best_response) == tuple(out.best_response):
        assert pol.value <= v_lp + 1e-5 * max(sc, 1.0)
    if storage == "f32":
        assert pol.value > out.best_value + 1e-7 or pol.point == 7


def test_polish_state_and_argument_errors():
    game = workloads.small_game(3, 3, 2, seed=5, kind="normal")
    with _make(game) as g:
        with pytest.raises(bsse.BsseError) as e:
            bsse.bsse_polish(g)
        assert e.value.status == bsse.BSSE_ESTATE
        bsse.bsse_lattice(g, 6)
        bsse.bsse_sweep(g)
        with pytest.raises(bsse.BsseError) as e:
            bsse.bsse_polish(g, profile=[0, 3])
        assert e.value.status == bsse.BSSE_EINVAL
        # a chunk swept since the last reported result: there is no completed sweep to polish
        for gm in (game, workloads.small_game(8, 8, 4, seed=6, kind="normal")):     # VALU and small-game paths
            with _make(gm) as h:
                bsse.bsse_lattice(h, 5)
                bsse.bsse_sweep(h)
                bsse.bsse_polish(h)
                bsse.bsse_sweep_chunk(h, None, 0, 0)
                with pytest.raises(bsse.BsseError) as e:
                    bsse.bsse_polish(h)
                assert e.value.status == bsse.BSSE_ESTATE
                bsse.bsse_sweep_result(h)
                bsse.bsse_polish(h)
                bsse.bsse_sweep_reset(h)
                with pytest.raises(bsse.BsseError) as e:
                    bsse.bsse_polish(h)
                assert e.value.status == bsse.BSSE_ESTATE


@pytest.mark.parametrize("shape,count", [((3, 3, 2), 4000), ((4, 3, 3), 20000), ((5, 4, 2), 20000),
                                         ((8, 8, 1), 20000)])
def test_solve_realised_equals_the_full_multiple_lps_solve(shape, count):
    """With a dense enough sweep the equilibrium's profile is realised by some candidate, and the
    solve over the realised profiles is the exact equilibrium value (the LP module enumerates all
    n^K profiles) at a fraction of the programs."""
    torch = _torch()
    m, n, K = shape
    game = workloads.small_game(m, n, K, seed=40 + m + n, kind="normal")
    v_sse, x_sse, prof_sse = sse_lp.solve(game.A, game.B, game.prior)
    X = workloads.host_candidates(m, count, seed=17, kind="dirichlet")
    with _make(game) as g:
        Xd = torch.from_numpy(X).cuda()
        sweep = bsse.bsse_sweep(g, Xd, count)
        v, x, prof, n_prof, n_solved = bsse.bsse_solve_realised(g, Xd, count)
    assert n_solved == n_prof <= n ** K
    assert sweep.best_value - 1e-6 <= v <= v_sse + 1e-8
    assert v == pytest.approx(v_sse, abs=1e-7 * max(1.0, abs(v_sse)))
    ok, v_ref, _ = sse_lp.profile_lp(game.A, game.B, game.prior, prof)
    assert ok and v == pytest.approx(v_ref, abs=1e-7 * max(1.0, abs(v_ref)))
    assert abs(float(x.sum()) - 1.0) < 1e-6 and (x >= 0).all()


def test_solve_realised_config1_and_truncation():
    game = workloads.game(1)
    v_sse, _, prof_sse = sse_lp.solve(game.A, game.B, game.prior)
    with _make(game) as g:
        bsse.bsse_lattice(g, 100)
        v, x, prof, n_prof, n_solved = bsse.bsse_solve_realised(g)
        assert v == pytest.approx(v_sse, abs=1e-8) and tuple(prof) == tuple(prof_sse)
        assert 1 <= n_prof <= 9 and n_solved == n_prof
        # one program only: the profile of the best swept candidate
        v1, _, prof1, n_prof1, n_solved1 = bsse.bsse_solve_realised(g, max_profiles=1)
        sweep = bsse.bsse_sweep(g)
        assert n_solved1 == 1 and n_prof1 == n_prof and tuple(prof1) == tuple(sweep.best_response)
        assert sweep.best_value - 1e-6 <= v1 <= v + 1e-12
