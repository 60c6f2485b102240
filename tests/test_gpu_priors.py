"""Prior-robustness batch (bsse_sweep_priors) against the oracle: for every prior of the batch the
result must be the sweep of the same game under that prior.  The oracle is simply run once per
prior; nothing here comes from the GPU path except what is being checked."""
import numpy as np
import pytest

from oracle import sweep as osweep
from paper_2605_18856_amd import bsse, workloads
from tests import parity
from tests.test_gpu_parity import _make, _run_eval

pytestmark = pytest.mark.gpu


def _priors(K, P, seed):
    """P priors: the K point masses first (as many as fit), then Dirichlet(1) draws and one
    uniform row; fp32 rows whose sum is within 1e-6 of 1."""
    rng = np.random.default_rng(seed)
    rows = [np.eye(K)[t] for t in range(min(K, max(P - 2, 0)))]
    while len(rows) < P - 1:
        rows.append(rng.dirichlet(np.ones(K)))
    rows.append(np.full(K, 1.0 / K))
    pri = np.asarray(rows[:P], dtype=np.float64)
    pri = (pri / pri.sum(axis=1, keepdims=True)).astype(np.float32)
    # fp32 rounding can leave the sum a few 1e-8 off; fix the largest entry
    for p in range(P):
        pri[p, np.argmax(pri[p])] += np.float32(1.0 - pri[p].astype(np.float64).sum())
    return pri


def _check_batch(game, X, pri, path=bsse.BSSE_PATH_AUTO, sample_only=False):
    tol = parity.TOL_BF16 if game.storage == "bf16" else parity.TOL_F32
    P, K = pri.shape
    with _make(game, path) as g:
        Xd, V_game, br_gpu = _run_eval(g, X)
        outs = bsse.bsse_sweep_priors(g, pri, Xd, X.shape[0])
        name = bsse.bsse_path_name(g)
        own = bsse.bsse_sweep(g, Xd, X.shape[0])
    assert len(outs) == P
    A, B, Xo = parity.oracle_inputs(game, X)
    exact_idx = 0
    for p in range(P):
        o = outs[p]
        assert 0 <= o.best_index < X.shape[0]
        assert o.n_evals == X.shape[0] * K
        # the winner's best responses are those the evaluation kernel reports for that row
        assert np.array_equal(o.best_response, br_gpu[o.best_index]), (p, name)
        # its value against the oracle's value of that row under the GPU's profile
        v_ref, sc = osweep.value_under_profile(A, pri[p], Xo[o.best_index].astype(np.float64),
                                               o.best_response)
        assert abs(o.best_value - v_ref) <= tol * max(sc, 1e-30), (p, o.best_value, v_ref)
        if sample_only:
            continue
        ref = osweep.sweep(A, B, pri[p], Xo, nthreads=8)
        # the oracle's own value at the GPU's winner is within tolerance of the oracle's optimum
        assert ref.values[o.best_index] >= ref.best_value - tol * max(sc, 1e-30), (p, name)
        exact_idx += int(o.best_index == ref.best_index)
    return outs, own, exact_idx


@pytest.mark.parametrize("shape,count,P", [((3, 3, 2), 700, 5), ((5, 7, 3), 1500, 9),
                                           ((8, 8, 4), 5000, 7), ((8, 8, 16), 3000, 20),
                                           ((16, 16, 8), 2500, 12), ((32, 32, 16), 3000, 70),
                                           ((32, 64, 6), 1200, 3)])
def test_prior_batch_against_oracle(shape, count, P):
    m, n, K = shape
    game = workloads.small_game(m, n, K, seed=77 + m + K, kind="normal")
    X = workloads.host_candidates(m, count, seed=5, kind="dirichlet")
    pri = _priors(K, P, seed=3)
    outs, own, exact = _check_batch(game, X, pri)
    assert exact >= P - max(1, P // 10)            # near-equal top values may swap the index


def test_prior_batch_forced_paths_and_bf16():
    game = workloads.small_game(32, 32, 8, seed=11, kind="normal")
    X = workloads.host_candidates(32, 2000, seed=6, kind="dirichlet")
    pri = _priors(8, 6, seed=4)
    for path in (bsse.BSSE_PATH_VALU, bsse.BSSE_PATH_MFMA, bsse.BSSE_PATH_MFMA_SPLIT):
        _check_batch(game, X, pri, path=path)
    gb = workloads.small_game(64, 128, 4, seed=12, kind="uniform", storage="bf16")
    Xb = workloads.host_candidates(64, 1500, seed=7, kind="dirichlet")
    _check_batch(gb, Xb, _priors(4, 5, seed=5))


def test_own_prior_reproduces_the_sweep_and_rows_are_independent():
    """A batch holding the game's own prior gives the sweep's answer: bit for bit on the paths that
    sum the types in the same order, within tolerance on the small-game kernel; and a prior's result
    does not depend on what else is in the batch."""
    for shape in ((5, 7, 3), (8, 8, 4), (32, 32, 16)):
        m, n, K = shape
        game = workloads.small_game(m, n, K, seed=31 + K, kind="normal")
        X = workloads.host_candidates(m, 4000, seed=8, kind="dirichlet")
        pri = _priors(K, 4, seed=9)
        pri[1] = game.prior
        outs, own, _ = _check_batch(game, X, pri)
        if (m, n) == (8, 8):
            assert abs(outs[1].best_value - own.best_value) <= 1e-5 * max(abs(own.best_value), 1e-3)
        else:
            assert outs[1].best_index == own.best_index
            assert np.float32(outs[1].best_value) == np.float32(own.best_value)
            assert np.array_equal(outs[1].best_response, own.best_response)
        with _make(game) as g:
            Xd, _, _ = _run_eval(g, X)
            solo = bsse.bsse_sweep_priors(g, pri[2:3], Xd, X.shape[0])[0]
        assert solo.best_index == outs[2].best_index
        assert np.float32(solo.best_value) == np.float32(outs[2].best_value)


def test_point_mass_prior_is_the_single_type_game():
    game = workloads.small_game(5, 7, 3, seed=90, kind="normal")
    X = workloads.host_candidates(5, 1000, seed=2, kind="dirichlet")
    pri = np.eye(3, dtype=np.float32)
    with _make(game) as g:
        Xd, _, _ = _run_eval(g, X)
        outs = bsse.bsse_sweep_priors(g, pri, Xd, X.shape[0])
    for t in range(3):
        ref = osweep.sweep(game.A[t:t + 1].copy(), game.B[t:t + 1].copy(), np.ones(1, np.float32), X,
                           nthreads=4)
        assert outs[t].best_index == ref.best_index
        assert abs(outs[t].best_value - ref.best_value) <= 1e-5 * max(abs(ref.best_value), 1e-3)
        assert outs[t].best_response[t] == ref.br[ref.best_index][0]


def test_exact_ties_in_a_batch():
    game = workloads.small_game(16, 16, 4, seed=21, kind="dup")
    X = workloads.host_candidates(16, 1500, seed=3, kind="dyadic")
    outs, _, _ = _check_batch(game, X, _priors(4, 6, seed=1))
    assert outs[0].n_tie_evals > 0


def test_argument_errors():
    game = workloads.small_game(3, 3, 2, seed=1, kind="normal")
    X = workloads.host_candidates(3, 10, seed=1, kind="dirichlet")
    with _make(game) as g:
        Xd, _, _ = _run_eval(g, X)
        bad = np.array([[0.5, 0.6]], dtype=np.float32)
        with pytest.raises(bsse.BsseError) as e:
            bsse.bsse_sweep_priors(g, bad, Xd, 10)
        assert e.value.status == bsse.BSSE_EINVAL
        nan = np.array([[np.nan, 1.0]], dtype=np.float32)
        with pytest.raises(bsse.BsseError) as e:
            bsse.bsse_sweep_priors(g, nan, Xd, 10)
        assert e.value.status == bsse.BSSE_ENOTFINITE
        ok = np.array([[0.25, 0.75]], dtype=np.float32)
        outs = bsse.bsse_sweep_priors(g, ok, Xd, 0)
        assert outs[0].best_index == -1 and outs[0].best_response is None


def test_large_game_more_than_one_chunk():
    """K = 256 caps a chunk of the leader-payoff matrix at 2^20 rows: 2^20 + 999 candidates take
    two chunks, the second one ragged.  Winners are checked one by one against the oracle."""
    import torch
    game = workloads.game(5)
    count = (1 << 20) + 999
    with _make(game) as g:
        Xd = torch.empty((count, game.m), dtype=torch.float32, device="cuda")
        bsse.bsse_dirichlet(g, 99, 0, count, Xd)
        pri = _priors(game.K, 3, seed=8)
        pri[0] = game.prior
        outs = bsse.bsse_sweep_priors(g, pri, Xd, count)
        own = bsse.bsse_sweep(g, Xd, count)
        torch.cuda.synchronize()
        rows = Xd[[o.best_index for o in outs]].cpu().numpy()
    assert outs[0].best_index == own.best_index
    assert np.float32(outs[0].best_value) == np.float32(own.best_value)
    for p, o in enumerate(outs):
        ref = osweep.sweep(game.A, game.B, pri[p], rows[p:p + 1], diagnostics=True, nthreads=8)
        mism = ref.br[0] != o.best_response
        assert not (mism & (ref.gap[0] >= 1e-6 * ref.scale[0])).any()
        v_ref, sc = osweep.value_under_profile(game.A, pri[p], rows[p].astype(np.float64), o.best_response)
        assert abs(o.best_value - v_ref) <= 1e-5 * max(sc, 1e-30)
