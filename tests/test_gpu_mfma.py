"""GPU parity tests of the matrix-core (MFMA) sweep kernels against the CPU oracle, through
the C ABI.  Small cases are compared element by element; the benchmark configurations are
run at full size in the launch shape bench.py times and compared on sampled candidates."""
import numpy as np
import pytest

from oracle import dirichlet as odir
from oracle import sweep as osweep
from paper_2605_18856_amd import bsse, workloads
from tests import parity
from tests.test_gpu_parity import _full_check, _make, _run_eval, _torch

pytestmark = pytest.mark.gpu

# (m, n, K, storage): every instantiated (m_pad, n) variant, with and without padding of m
# and of the type count
MFMA_SHAPES = [
    (8, 8, 4, "f32"), (8, 8, 3, "f32"), (5, 8, 9, "f32"),
    (8, 8, 8, "f32"), (6, 8, 12, "f32"), (8, 8, 16, "f32"), (3, 8, 4, "f32"),
    (16, 16, 3, "f32"), (12, 16, 2, "f32"),
    (32, 32, 16, "f32"), (20, 32, 5, "f32"),
    (32, 64, 3, "f32"), (24, 64, 2, "f32"),
    (128, 256, 2, "f32"), (100, 256, 1, "f32"),
    (16, 32, 3, "bf16"), (32, 16, 5, "bf16"), (9, 32, 2, "bf16"),
    (64, 128, 4, "bf16"), (50, 128, 2, "bf16"),
    # the wide bf16 game with many types (several stages per launch) and a padded m
    (64, 128, 8, "bf16"), (64, 128, 24, "bf16"), (50, 128, 16, "bf16"),
]


@pytest.mark.parametrize("shape", MFMA_SHAPES, ids=lambda s: "m%dn%dK%d%s" % s)
@pytest.mark.parametrize("count", [1, 33, 1300, 70001])
def test_mfma_path_parity(shape, count):
    m, n, K, storage = shape
    game = workloads.small_game(m, n, K, 500 + m + n + K, kind="normal", storage=storage)
    X = workloads.host_candidates(m, count, 11 + count, "dirichlet")
    _full_check(game, X, bsse.BSSE_PATH_MFMA, "mfma")


# (m, n, K, payoff kind): the split path (bf16 matrix cores on fp32 operands cut into bf16 parts);
# integer payoffs are bf16 numbers and take the three-term variant, the others six terms
SPLIT_SHAPES = [
    (16, 16, 3, "normal"), (12, 16, 2, "normal"), (32, 32, 16, "normal"), (20, 32, 5, "normal"),
    (32, 64, 3, "normal"), (24, 64, 2, "uniform"), (32, 32, 4, "int"), (128, 256, 2, "int"),
    (100, 256, 1, "int"),
]


@pytest.mark.parametrize("shape", SPLIT_SHAPES, ids=lambda s: "m%dn%dK%d%s" % s)
@pytest.mark.parametrize("count", [1, 33, 1300, 70001])
def test_split_path_parity(shape, count):
    m, n, K, kind = shape
    game = workloads.small_game(m, n, K, 900 + m + n + K, kind=kind)
    X = workloads.host_candidates(m, count, 13 + count, "dirichlet")
    expect = "mfma_split3" if kind == "int" else "mfma_split6"
    _full_check(game, X, bsse.BSSE_PATH_MFMA_SPLIT, expect)


@pytest.mark.parametrize("shape", [(32, 32, 3), (32, 64, 2), (128, 256, 1)], ids=lambda s: "m%dn%dK%d" % s)
@pytest.mark.parametrize("kind", ["dyadic", "vertex"])
def test_split_exact_ties(shape, kind):
    m, n, K = shape
    game = workloads.small_game(m, n, K, 79, kind="dup")
    X = workloads.host_candidates(m, 700, 80, kind)
    # integer payoffs are bf16 numbers: three terms where the shape has such a variant
    rep, out = _full_check(game, X, bsse.BSSE_PATH_MFMA_SPLIT, "mfma_split6" if n == 64 else "mfma_split3")
    assert rep.br_mismatch == 0
    ref = osweep.sweep(game.A, game.B, game.prior, X, diagnostics=True)
    assert out.n_tie_evals == int((ref.gap == 0).sum()) > 0


def test_split_path_rejects_what_it_cannot_do():
    g8 = workloads.small_game(8, 9, 2, 1)
    with pytest.raises(bsse.BsseError) as e:
        bsse.bsse_create(8, 9, 2, g8.A, g8.B, g8.prior, path=bsse.BSSE_PATH_MFMA_SPLIT)
    assert e.value.status == bsse.BSSE_EINVAL
    gb = workloads.small_game(32, 32, 2, 1)
    with pytest.raises(bsse.BsseError) as e:
        bsse.bsse_create(32, 32, 2, gb.A, gb.B, gb.prior, storage=bsse.BSSE_STORAGE_BF16,
                         path=bsse.BSSE_PATH_MFMA_SPLIT)
    assert e.value.status == bsse.BSSE_EINVAL
    # a real-valued 128x256 game has no six-term variant: forced split fails, AUTO falls back
    gr = workloads.small_game(128, 256, 1, 2)
    with pytest.raises(bsse.BsseError):
        bsse.bsse_create(128, 256, 1, gr.A, gr.B, gr.prior, path=bsse.BSSE_PATH_MFMA_SPLIT)
    with bsse.bsse_create(128, 256, 1, gr.A, gr.B, gr.prior) as g:
        assert bsse.bsse_path_name(g) == "mfma_f32"


@pytest.mark.parametrize("shape", [(8, 8, 5, "f32"), (8, 8, 4, "f32"), (7, 8, 8, "f32"), (16, 16, 3, "f32"), (32, 32, 3, "f32"),
                                   (32, 64, 2, "f32"), (16, 32, 3, "bf16"), (64, 128, 2, "bf16"),
                                   (64, 128, 8, "bf16"), (33, 128, 16, "bf16")],
                         ids=lambda s: "m%dn%dK%d%s" % s)
@pytest.mark.parametrize("kind", ["dyadic", "vertex"])
def test_mfma_exact_ties(shape, kind):
    """Integer payoffs with duplicated follower columns and exactly representable candidates:
    every product and partial sum is exact in any order, so both sides see the same ties and
    best responses must agree with no exception."""
    m, n, K, storage = shape
    game = workloads.small_game(m, n, K, 77, kind="dup", storage=storage)
    X = workloads.host_candidates(m, 700, 78, kind)
    rep, out = _full_check(game, X, bsse.BSSE_PATH_MFMA, "mfma")
    assert rep.br_mismatch == 0
    ref = osweep.sweep(game.A, game.B, game.prior, X, diagnostics=True)
    assert (ref.gap == 0).sum() > 0
    assert out.n_tie_evals == int((ref.gap == 0).sum())


def test_mfma_and_valu_paths_agree_on_hand_cases():
    """2x2 hand game embedded in an 8x8 shape: the tie-break decides the optimum."""
    A = np.zeros((1, 8, 8), np.float32)
    B = np.full((1, 8, 8), -5.0, np.float32)
    A[0, :2, :2] = [[2, 4], [1, 3]]
    B[0, :2, :2] = [[1, 0], [0, 1]]
    X = np.zeros((101, 8), np.float32)
    X[:, 0] = np.arange(101) / np.float32(100)
    X[:, 1] = np.float32(1) - X[:, 0]
    for path in (bsse.BSSE_PATH_VALU, bsse.BSSE_PATH_MFMA):
        with bsse.bsse_create(8, 8, 1, A, B, np.array([1.0], np.float32), path=path) as g:
            Xd = _torch().from_numpy(X).cuda()
            out = bsse.bsse_sweep(g, Xd, 101)
            assert out.best_index == 50 and out.best_value == 3.5 and out.best_response[0] == 1


def _sampled_check(game, count, sample_rows, chunk=None):
    """Full-size run in bench.py's launch shape; oracle on a sample of rows + the winner."""
    torch = _torch()
    tol = parity.TOL_BF16 if game.storage == "bf16" else parity.TOL_F32
    with _make(game) as g:
        assert bsse.bsse_path_name(g).startswith("mfma")
        Xd = torch.empty((count, game.m), dtype=torch.float32, device="cuda")
        bsse.bsse_dirichlet(g, game.candidate_seed, 0, count, Xd)
        V = torch.empty(count, dtype=torch.float32, device="cuda")
        br = torch.empty((count, game.K), dtype=torch.int32, device="cuda")
        bsse.bsse_eval(g, Xd, count, V, br)
        out = bsse.bsse_sweep(g, Xd, count)
        torch.cuda.synchronize()
        # reduction: CPU arg-max (first maximum) over the GPU's own values, bit-exact
        Vh = V.cpu().numpy()
        c_cpu = int(np.argmax(Vh))
        assert out.best_index == c_cpu and np.float32(out.best_value) == Vh[c_cpu]
        rows = np.unique(np.concatenate([np.arange(min(sample_rows // 2, count)),
                                         np.linspace(0, count - 1, sample_rows // 2).astype(np.int64),
                                         [out.best_index]]))
        idx = torch.from_numpy(rows).cuda()
        Xs = Xd[idx].cpu().numpy()
        rep = parity.compare_eval(game, Xs, Vh[rows], br[idx].cpu().numpy(), tol)
        parity.check_report(rep, tol)
        assert np.array_equal(out.best_response, br[out.best_index].cpu().numpy())
        if chunk:
            bsse.bsse_sweep_reset(g)
            for a in range(0, count, chunk):
                b = min(count, a + chunk)
                bsse.bsse_sweep_chunk(g, Xd[a:b], b - a, a)
            parts = bsse.bsse_sweep_result(g)
            assert (parts.best_index, parts.best_value) == (out.best_index, out.best_value)
        return rep


def test_config2_full_size():
    rep = _sampled_check(workloads.game(2), 1 << 20, 1 << 16, chunk=(1 << 18) + 3)
    assert rep.n_evals >= (1 << 16) * 4 // 2


def test_config3_full_size_sampled():
    _sampled_check(workloads.game(3), 1 << 24, 8192)


def test_config3_fp32_mfma_path_sampled():
    """The plain fp32 MFMA kernel stays reachable and correct when forced."""
    game = workloads.game(3)
    X = workloads.host_candidates(game.m, 3000, 5, "dirichlet")
    _full_check(game, X, bsse.BSSE_PATH_MFMA, "mfma_f32")


def test_config4_one_chunk_sampled():
    _sampled_check(workloads.game(4), 1 << 22, 8192)


def test_config5_subrange_sampled():
    _sampled_check(workloads.game(5), 1 << 16, 4096)


def test_config5_tie_injected_variant():
    """Duplicated follower columns at the benchmark shape: the leader-favourable rule and the
    lowest-index rule decide a large share of the evaluations."""
    game = workloads.game(5, "ties")
    torch = _torch()
    count = 384
    X = np.concatenate([workloads.host_candidates(game.m, count - 128, 5, "dirichlet"),
                        workloads.host_candidates(game.m, 64, 6, "vertex"),
                        workloads.host_candidates(game.m, 64, 7, "dyadic")])
    with _make(game) as g:
        Xd, V, br = _run_eval(g, X)
        rep = parity.compare_eval(game, X, V, br)
        parity.check_report(rep, parity.TOL_F32)
        out = bsse.bsse_sweep(g, Xd, count)
        ref = osweep.sweep(game.A, game.B, game.prior, X[-128:], diagnostics=True, nthreads=8)
        # exactly representable candidates: ties are exact on both sides, so are the answers
        assert np.array_equal(br[-128:], ref.br)
        assert (ref.gap == 0).sum() > 1000
        assert out.n_tie_evals >= int((ref.gap == 0).sum())


def _full_streamed(game, total, chunk):
    """The whole configured candidate count, streamed in bench.py's chunks (generate a chunk of the
    seeded sequence, sweep it, merge): n_evals covers everything; the winner, regenerated from its
    index alone, is checked against the oracle (its value under the reported profile, and the
    oracle's own best responses at that row up to flagged near-ties); every chunk's own best is no
    better than the overall best."""
    torch = _torch()
    tol = parity.TOL_BF16 if game.storage == "bf16" else parity.TOL_F32
    seed = game.candidate_seed
    with _make(game) as g:
        Xd = torch.empty((chunk, game.m), dtype=torch.float32, device="cuda")
        bsse.bsse_sweep_reset(g)
        for base in range(0, total, chunk):
            bsse.bsse_dirichlet(g, seed, base, chunk, Xd)
            bsse.bsse_sweep_chunk(g, Xd, chunk, base)
        out = bsse.bsse_sweep_result(g)
        assert out.n_evals == total * game.K and 0 <= out.best_index < total
        row_dev = torch.empty((1, game.m), dtype=torch.float32, device="cuda")
        bsse.bsse_dirichlet(g, seed, out.best_index, 1, row_dev)
        torch.cuda.synchronize()
        row = row_dev.cpu().numpy()
        assert np.array_equal(bsse.bsse_sweep_best_row(g), row[0])
        # the chunk that holds the winner, swept alone, gives the same answer
        base = out.best_index // chunk * chunk
        bsse.bsse_dirichlet(g, seed, base, chunk, Xd)
        alone = bsse.bsse_sweep(g, Xd, chunk)
        assert alone.best_index + base == out.best_index
        assert np.float32(alone.best_value) == np.float32(out.best_value)
    # the oracle makes the winning row itself, from the index alone
    row_o = odir.rows(seed, out.best_index, 1, game.m).astype(np.float32)
    assert np.allclose(row, row_o, rtol=4e-6, atol=1e-9)
    A, B, Xo = parity.oracle_inputs(game, row_o)
    ref = osweep.sweep(A, B, game.prior, Xo, diagnostics=True, nthreads=8)
    mism = ref.br[0] != out.best_response
    assert not (mism & (ref.gap[0] >= 1e-6 * ref.scale[0])).any()
    v_ref, sc = osweep.value_under_profile(A, game.prior, Xo[0].astype(np.float64), out.best_response)
    assert abs(out.best_value - v_ref) <= tol * max(sc, 1e-30)
    return out


def _range_sample(game, total, winner, n_first=4096, n_strided=4096, bound_budget=0):
    """Per-candidate parity on a sample of the whole configured range: the first n_first rows, n_strided
    rows spread evenly over all `total`, and the sweep's winner; each row is made by the device
    generator from its global index, evaluated with per-candidate outputs, and compared with the
    oracle on those same row bits."""
    torch = _torch()
    tol = parity.TOL_BF16 if game.storage == "bf16" else parity.TOL_F32
    rows = np.unique(np.concatenate([np.arange(n_first), np.linspace(0, total - 1, n_strided).astype(np.int64),
                                     [winner.best_index]]))
    with _make(game) as g:
        Xs = torch.empty((len(rows), game.m), dtype=torch.float32, device="cuda")
        bsse.bsse_dirichlet(g, game.candidate_seed, 0, n_first, Xs)
        for q in range(n_first, len(rows)):
            bsse.bsse_dirichlet(g, game.candidate_seed, int(rows[q]), 1, Xs[q:q + 1])
        V = torch.empty(len(rows), dtype=torch.float32, device="cuda")
        br = torch.empty((len(rows), game.K), dtype=torch.int32, device="cuda")
        bsse.bsse_eval(g, Xs, len(rows), V, br)
        torch.cuda.synchronize()
        Vh, brh = V.cpu().numpy(), br.cpu().numpy()
        rep = parity.compare_eval(game, Xs.cpu().numpy(), Vh, brh, tol)
        parity.check_report(rep, tol, bound_budget, label=game.name)
        # the winner's per-candidate value and best responses are what the sweep reported
        w = int(np.searchsorted(rows, winner.best_index))
        assert np.float32(winner.best_value) == Vh[w] and np.array_equal(winner.best_response, brh[w])
        # and no sampled candidate beats it
        assert Vh.max() <= np.float32(winner.best_value)
    return rep


def test_config4_all_sixteen_chunks():
    game = workloads.game(4)
    out = _full_streamed(game, 1 << 26, 1 << 22)
    rep = _range_sample(game, 1 << 26, out)
    assert rep.n_evals >= 8000 * game.K


def test_config5_whole_range():
    game = workloads.game(5)
    out = _full_streamed(game, 1 << 24, 1 << 20)
    rep = _range_sample(game, 1 << 24, out)
    assert rep.n_evals >= 8000 * game.K


def test_config3_whole_range_against_the_oracle():
    """Config 3 is small enough for the oracle to sweep all 2^24 candidates (about 10^12 fp64
    operations): every per-candidate value and best response is compared, and the sweep's winner
    with the oracle's own arg-max over the whole range."""
    torch = _torch()
    game = workloads.game(3)
    total, piece = 1 << 24, 1 << 21
    tol = parity.TOL_F32
    best = (-np.inf, -1)
    with _make(game) as g:
        Xd = torch.empty((total, game.m), dtype=torch.float32, device="cuda")
        bsse.bsse_dirichlet(g, game.candidate_seed, 0, total, Xd)
        V = torch.empty(total, dtype=torch.float32, device="cuda")
        br = torch.empty((total, game.K), dtype=torch.int32, device="cuda")
        bsse.bsse_eval(g, Xd, total, V, br)
        out = bsse.bsse_sweep(g, Xd, total)
        torch.cuda.synchronize()
        Vh = V.cpu().numpy()
        assert out.best_index == int(np.argmax(Vh)) and np.float32(out.best_value) == Vh[out.best_index]
        flagged = bound = 0
        for a in range(0, total, piece):
            Xp = Xd[a:a + piece].cpu().numpy()
            brp = br[a:a + piece].cpu().numpy()
            ref = osweep.sweep(game.A, game.B, game.prior, Xp, diagnostics=True, nthreads=16)
            rep = parity.compare_eval(game, Xp, Vh[a:a + piece], brp, tol, nthreads=16, ref=ref)
            parity.check_report(rep, tol, bound_budget=0, label="config3 rows %d.." % a)
            flagged += rep.flagged
            if ref.best_value > best[0]:
                best = (ref.best_value, a + ref.best_index)
            print("config3 rows %d..%d compared, flagged so far %d" % (a, a + piece, flagged), flush=True)
        # the oracle's value at the GPU's winner is within tolerance of the oracle's optimum
        Xw = Xd[out.best_index:out.best_index + 1].cpu().numpy()
        rw = osweep.sweep(game.A, game.B, game.prior, Xw, diagnostics=True)
        _, sc = osweep.value_under_profile(game.A, game.prior, Xw[0].astype(np.float64), rw.best_br)
        assert rw.best_value >= best[0] - tol * sc
        print("config3 whole range: gpu winner %d, oracle winner %d, flagged %d of %d evaluations"
              % (out.best_index, best[1], flagged, total * game.K), flush=True)
