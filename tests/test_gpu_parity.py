"""GPU parity tests: every call goes through the C ABI (via the ctypes binding) and is
compared element by element with the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

from oracle import dirichlet as odir
from oracle import lattice as olat
from oracle import sse_lp
from oracle import sweep as osweep
from paper_2605_18856_amd import bsse, workloads
from tests import parity

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def _run_eval(g, X):
    torch = _torch()
    Xd = torch.from_numpy(np.ascontiguousarray(X, dtype=np.float32)).cuda()
    C = X.shape[0]
    V = torch.empty(C, dtype=torch.float32, device="cuda")
    br = torch.empty((C, g.K), dtype=torch.int32, device="cuda")
    bsse.bsse_eval(g, Xd, C, V, br)
    torch.cuda.synchronize()
    return Xd, V.cpu().numpy(), br.cpu().numpy()


def _make(game, path=bsse.BSSE_PATH_AUTO):
    storage = bsse.BSSE_STORAGE_BF16 if game.storage == "bf16" else bsse.BSSE_STORAGE_F32
    return bsse.bsse_create(game.m, game.n, game.K, game.A, game.B, game.prior,
                            storage=storage, path=path)


def _full_check(game, X, path=bsse.BSSE_PATH_AUTO, expect_path=None):
    tol = parity.TOL_BF16 if game.storage == "bf16" else parity.TOL_F32
    with _make(game, path) as g:
        if expect_path:
            assert bsse.bsse_path_name(g).startswith(expect_path)
        Xd, V, br = _run_eval(g, X)
        rep = parity.compare_eval(game, X, V, br, tol)
        parity.check_report(rep, tol)
        out = bsse.bsse_sweep(g, Xd, X.shape[0])
        assert out.n_evals == X.shape[0] * game.K
        parity.check_winner(game, X, out, V, tol)
        assert np.array_equal(out.best_response, br[out.best_index])
        return rep, out


# ------------------------------------------------------------------ config 1: lattice + LP
def test_config1_lattice_sweep_against_oracle_and_lp():
    game = workloads.game(1)
    with _make(game) as g:
        count = bsse.bsse_lattice(g, 100)
        assert count == 5151
        X = bsse.candidates_to_host(g)
        assert np.array_equal(X, olat.points_f32(3, 100))         # bit-exact lattice
        out = bsse.bsse_sweep(g)                                   # the generated set
        ref = osweep.sweep(game.A, game.B, game.prior, X)
        assert out.best_index == ref.best_index
        assert np.array_equal(out.best_response, ref.best_br)
        assert abs(out.best_value - ref.best_value) <= 1e-5
        v_lp, _, _ = sse_lp.solve(game.A, game.B, game.prior)
        assert out.best_value <= v_lp + 1e-5 and v_lp - out.best_value <= 0.12
        Xd, V, br = _run_eval(g, X)
        parity.check_report(parity.compare_eval(game, X, V, br), parity.TOL_F32)


@pytest.mark.parametrize("m,N", [(1, 7), (2, 50), (3, 17), (4, 9), (5, 6), (8, 4)])
def test_lattice_bit_exact(m, N):
    game = workloads.small_game(m, 3, 1, 5)
    with _make(game) as g:
        count = bsse.bsse_lattice(g, N)
        assert count == olat.count(m, N)
        assert np.array_equal(bsse.candidates_to_host(g), olat.points_f32(m, N))


def test_hand_2x2_tiebreak_on_gpu():
    A = np.array([[[2, 4], [1, 3]]], np.float32)
    B = np.array([[[1, 0], [0, 1]]], np.float32)
    with bsse.bsse_create(2, 2, 1, A, B, np.array([1.0], np.float32)) as g:
        for N, val, k0 in [(2, 3.5, 1), (10, 3.5, 5), (100, 3.5, 50), (3, 10 / 3, 1), (7, 24 / 7, 3)]:
            assert bsse.bsse_lattice(g, N) == N + 1
            out = bsse.bsse_sweep(g)
            assert out.best_value == pytest.approx(val, rel=1e-6)
            assert out.best_index == k0
            assert out.best_response[0] == 1
            if N % 2 == 0:
                assert out.n_tie_evals >= 1


# ------------------------------------------------------------------------- Dirichlet rows
@pytest.mark.parametrize("m", [3, 8, 32, 64, 128, 6, 12])
def test_dirichlet_rows_against_oracle(m):
    torch = _torch()
    game = workloads.small_game(m, 2, 1, 1)
    seed, first, count = 3000 + m, (1 << 32) - 700, 1500      # crosses the 32-bit row index
    with _make(game) as g:
        out = torch.empty((count, m), dtype=torch.float32, device="cuda")
        bsse.bsse_dirichlet(g, seed, first, count, out)
        torch.cuda.synchronize()
        X = out.cpu().numpy()
        ref = odir.rows(seed, first, count, m)
        assert np.all(X >= 0) and np.allclose(X.sum(1, dtype=np.float64), 1.0, atol=2e-6)
        assert np.allclose(X, ref, rtol=2e-6, atol=1e-9)
        # chunking and handle-owned buffer give the same bits
        bsse.bsse_dirichlet(g, seed, first + 500, 1000)
        assert np.array_equal(bsse.candidates_to_host(g), X[500:])


@pytest.mark.parametrize("m", [4, 8, 32, 64, 256])
def test_dirichlet_rows_do_not_depend_on_output_alignment(m):
    """An output buffer that is only 4-byte aligned takes another generation kernel; the rows are
    the same bits (row c is a function of the seed and c alone)."""
    torch = _torch()
    game = workloads.small_game(m, 2, 1, 1)
    seed, first, count = 77, 12345, 777
    with _make(game) as g:
        aligned = torch.empty((count, m), dtype=torch.float32, device="cuda")
        flat = torch.zeros(count * m + 4, dtype=torch.float32, device="cuda")
        bsse.bsse_dirichlet(g, seed, first, count, aligned)
        for off in (1, 2, 3):
            view = flat[off:off + count * m]
            assert view.data_ptr() % 16 != 0
            bsse.bsse_dirichlet(g, seed, first, count, view)
            torch.cuda.synchronize()
            assert torch.equal(view.view(count, m), aligned)


# --------------------------------------------------------------------- VALU path, shapes
VALU_SHAPES = [(3, 3, 2), (8, 8, 4), (5, 7, 3), (1, 4, 2), (4, 1, 3), (16, 33, 2), (70, 9, 2),
               (300, 5, 2)]


@pytest.mark.parametrize("shape", VALU_SHAPES)
@pytest.mark.parametrize("count", [1, 63, 64, 1000])
def test_valu_path_parity(shape, count):
    m, n, K = shape
    game = workloads.small_game(m, n, K, 100 + m + n + K, kind="normal")
    X = workloads.host_candidates(m, count, 7 + count, "dirichlet")
    _full_check(game, X, bsse.BSSE_PATH_VALU, "valu")


@pytest.mark.parametrize("kind", ["dyadic", "vertex", "sparse"])
def test_valu_path_exact_ties(kind):
    """Duplicated follower columns and integer payoffs: exact ties on both sides."""
    game = workloads.small_game(6, 10, 3, 31, kind="dup")
    X = workloads.host_candidates(6, 500, 32, kind)
    rep, out = _full_check(game, X, bsse.BSSE_PATH_VALU, "valu")
    assert rep.br_mismatch == 0 or kind == "sparse"
    ref = osweep.sweep(game.A, game.B, game.prior, X, diagnostics=True)
    assert (ref.gap == 0).sum() > 0
    if kind != "sparse":
        assert out.n_tie_evals == int((ref.gap == 0).sum())


def test_valu_bf16_storage():
    game = workloads.small_game(16, 24, 3, 41, kind="uniform", storage="bf16")
    # payoffs that are NOT yet bf16 values: the library rounds them itself
    raw = workloads.small_game(16, 24, 3, 41, kind="uniform")
    X = workloads.host_candidates(16, 700, 42, "dirichlet")
    with bsse.bsse_create(16, 24, 3, raw.A, raw.B, raw.prior, storage=bsse.BSSE_STORAGE_BF16,
                          path=bsse.BSSE_PATH_VALU) as g:
        Xd, V, br = _run_eval(g, X)
        parity.check_report(parity.compare_eval(game, X, V, br, parity.TOL_BF16), parity.TOL_BF16)


def test_config2_subset_and_chunking():
    torch = _torch()
    game = workloads.game(2)
    count = (1 << 14) + 37
    with _make(game) as g:
        Xd = torch.empty((count, game.m), dtype=torch.float32, device="cuda")
        bsse.bsse_dirichlet(g, game.candidate_seed, 0, count, Xd)
        torch.cuda.synchronize()
        X = Xd.cpu().numpy()
        V = torch.empty(count, dtype=torch.float32, device="cuda")
        br = torch.empty((count, game.K), dtype=torch.int32, device="cuda")
        bsse.bsse_eval(g, Xd, count, V, br)
        torch.cuda.synchronize()
        Vh, brh = V.cpu().numpy(), br.cpu().numpy()
        parity.check_report(parity.compare_eval(game, X, Vh, brh), parity.TOL_F32)
        whole = bsse.bsse_sweep(g, Xd, count)
        parity.check_winner(game, X, whole, Vh)
        # streamed in ragged chunks: same winner, same value, same best responses
        bsse.bsse_sweep_reset(g)
        edges = [0, 1, 65, 4096, 9000, count]
        for a, b in zip(edges[:-1], edges[1:]):
            bsse.bsse_sweep_chunk(g, Xd[a:b], b - a, a)
        parts = bsse.bsse_sweep_result(g)
        assert (parts.best_index, parts.best_value) == (whole.best_index, whole.best_value)
        assert np.array_equal(parts.best_response, whole.best_response)
        assert parts.n_evals == whole.n_evals == count * game.K


def test_duplicate_candidates_keep_lowest_index_across_chunks():
    torch = _torch()
    game = workloads.small_game(4, 5, 2, 9)
    X = workloads.host_candidates(4, 300, 10)
    X2 = np.concatenate([X, X, X])
    with _make(game) as g:
        Xd = torch.from_numpy(X2).cuda()
        one = bsse.bsse_sweep(g, Xd[:300].contiguous(), 300)
        three = bsse.bsse_sweep(g, Xd, 900)
        assert three.best_index == one.best_index and three.best_value == one.best_value
        bsse.bsse_sweep_reset(g)
        for k in range(3):
            bsse.bsse_sweep_chunk(g, Xd[300 * k:300 * (k + 1)], 300, 300 * k)
        assert bsse.bsse_sweep_result(g).best_index == one.best_index


def test_empty_inputs_and_state_errors():
    torch = _torch()
    game = workloads.small_game(4, 5, 2, 9)
    with _make(game) as g:
        with pytest.raises(bsse.BsseError) as e:
            bsse.bsse_sweep(g)                      # nothing generated yet
        assert e.value.status == bsse.BSSE_ESTATE
        empty = torch.zeros((1, 4), dtype=torch.float32, device="cuda")   # a real pointer, 0 rows used
        out = bsse.bsse_sweep(g, empty, 0)
        assert out.best_index == -1 and out.best_response is None and out.n_evals == 0
        bsse.bsse_eval(g, empty, 0, None, None)
        assert bsse.lib().bsse_sweep_chunk(g.handle, empty.data_ptr(), -1, 0) == bsse.BSSE_EINVAL
        assert bsse.lib().bsse_sweep_chunk(g.handle, empty.data_ptr(), 0, -5) == bsse.BSSE_EINVAL
        with pytest.raises(bsse.BsseError) as e:
            bsse.bsse_lattice(g, 100000)            # 4 parts, N=1e5: > 2^40 points
        assert e.value.status == bsse.BSSE_EOVERFLOW


def test_timing_counters():
    torch = _torch()
    game = workloads.game(2)
    with _make(game) as g:
        Xd = torch.empty((4096, game.m), dtype=torch.float32, device="cuda")
        bsse.bsse_dirichlet(g, 1, 0, 4096, Xd)
        bsse.bsse_set_timing(g, True)
        for _ in range(3):
            bsse.bsse_sweep(g, Xd, 4096)
        ms, launches = bsse.bsse_get_timing(g)
        assert launches == 3 and ms > 0
