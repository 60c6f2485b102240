"""bsse_sweep_dirichlet: the sweep over seeded flat-Dirichlet rows that are never written out.

Two kinds of check.  Against the library's own two-step form (bsse_dirichlet into a buffer, then
bsse_sweep): the contract is equality bit for bit, on every shape family.  Against the oracle: the
oracle generates the rows itself (fp64 generator, rounded to fp32) and sweeps them; the library's
winner must be the oracle's up to near-equal values, and its value must be the oracle's value of
that row within tolerance."""
import numpy as np
import pytest

from oracle import dirichlet as odir
from oracle import sweep as osweep
from paper_2605_18856_amd import bsse, workloads
from tests import parity
from tests.test_gpu_parity import _make

pytestmark = pytest.mark.gpu


def _two_step(g, seed, first, count):
    """(outcome, winning row) of generate-then-sweep; the row as the handle reports it must be the
    row of the buffer at best_index"""
    import torch
    X = torch.empty((max(count, 1), g.m), dtype=torch.float32, device="cuda")
    bsse.bsse_dirichlet(g, seed, first, count, X)
    out = bsse.bsse_sweep(g, X, count)
    torch.cuda.synchronize()
    row = X[out.best_index].cpu().numpy()
    assert np.array_equal(bsse.bsse_sweep_best_row(g), row)
    return out, row


def _fused(g, seed, first, count):
    out = bsse.bsse_sweep_dirichlet(g, seed, first, count)
    return out, bsse.bsse_sweep_best_row(g)


def _same(a, b):
    if isinstance(a, tuple):
        assert np.array_equal(a[1], b[1])             # the winning row, bit for bit
        a, b = a[0], b[0]
    assert a.best_index == b.best_index
    assert np.float32(a.best_value) == np.float32(b.best_value)
    assert a.n_evals == b.n_evals and a.n_tie_evals == b.n_tie_evals
    if a.best_index >= 0:
        assert np.array_equal(a.best_response, b.best_response)


@pytest.mark.parametrize("K", [4, 8, 12, 16])
def test_small_game_fused_equals_two_step(K):
    game = workloads.small_game(8, 8, K, seed=40 + K, kind="normal")
    with _make(game) as g:
        assert bsse.bsse_path_name(g).startswith("mfma")
        for seed, first, count in [(1, 0, 1), (2, 0, 31), (3, 7, 64), (4, 12345, 65), (5, 0, 1000),
                                   (6, (1 << 32) - 100, 777), (7, 3, (1 << 17) + 5),
                                   ((1 << 63) + 12345, (1 << 40) + 1, 50000)]:
            _same(_fused(g, seed, first, count), _two_step(g, seed, first, count))


@pytest.mark.parametrize("shape,storage", [((3, 3, 2), "f32"), ((5, 7, 3), "f32"), ((16, 16, 8), "f32"),
                                           ((32, 32, 16), "f32"), ((64, 128, 4), "bf16")])
def test_other_shapes_equal_two_step(shape, storage):
    m, n, K = shape
    game = workloads.small_game(m, n, K, seed=9 + m, kind="normal" if storage == "f32" else "uniform",
                                storage=storage)
    with _make(game) as g:
        for seed, first, count in [(11, 0, 1), (12, 5, 999), (13, 1 << 33, 40000)]:
            _same(_fused(g, seed, first, count), _two_step(g, seed, first, count))


def test_staged_pieces_and_chunks():
    """m = 16: a staging piece holds 2^22 rows, so 2^22 + 4097 rows take two pieces; and the streamed
    form in three unequal chunks gives the one-shot result (global indices, strict merge)."""
    game = workloads.small_game(16, 16, 4, seed=3, kind="normal")
    count = (1 << 22) + 4097
    with _make(game) as g:
        one = bsse.bsse_sweep_dirichlet(g, 21, 10, count)
        _same((one, bsse.bsse_sweep_best_row(g)), _two_step(g, 21, 10, count))
        bsse.bsse_sweep_reset(g)
        cuts = [0, 1000, (1 << 22) - 3, count]
        for lo, hi in zip(cuts[:-1], cuts[1:]):
            bsse.bsse_sweep_dirichlet_chunk(g, 21, 10 + lo, hi - lo, lo)
        _same(bsse.bsse_sweep_result(g), one)
    small = workloads.game(2)
    with _make(small) as g:
        one = bsse.bsse_sweep_dirichlet(g, 5, 0, 300000)
        bsse.bsse_sweep_reset(g)
        for lo, hi in [(0, 70001), (70001, 70002), (70002, 300000)]:
            bsse.bsse_sweep_dirichlet_chunk(g, 5, lo, hi - lo, lo)
        _same(bsse.bsse_sweep_result(g), one)


@pytest.mark.parametrize("shape", [(8, 8, 4), (8, 8, 16), (3, 3, 2), (16, 16, 8)])
def test_chunk_order_does_not_matter_and_equal_values_keep_the_lowest_index(shape):
    """The same rows submitted as several chunks, in any order: the result is that of one sweep in
    index order.  Submitting one buffer twice under two index bases makes every value occur twice:
    the copy with the lower global index must win."""
    import torch
    m, n, K = shape
    game = workloads.small_game(m, n, K, seed=60 + K, kind="normal")
    count = 50000
    with _make(game) as g:
        X = torch.empty((count, m), dtype=torch.float32, device="cuda")
        bsse.bsse_dirichlet(g, 31, 0, count, X)
        one = bsse.bsse_sweep(g, X, count)
        cuts = [0, 12345, 12346, 40000, count]
        spans = list(zip(cuts[:-1], cuts[1:]))
        for order in (spans, spans[::-1], [spans[2], spans[0], spans[3], spans[1]]):
            bsse.bsse_sweep_reset(g)
            for lo, hi in order:
                bsse.bsse_sweep_chunk(g, X[lo:hi], hi - lo, lo)
            _same(bsse.bsse_sweep_result(g), one)
            bsse.bsse_sweep_reset(g)
            for lo, hi in order:
                bsse.bsse_sweep_dirichlet_chunk(g, 31, lo, hi - lo, lo)
            _same(bsse.bsse_sweep_result(g), one)
        for bases in ((0, count), (count, 0)):
            bsse.bsse_sweep_reset(g)
            for b in bases:
                bsse.bsse_sweep_chunk(g, X, count, b)
            twice = bsse.bsse_sweep_result(g)
            assert twice.best_index == one.best_index
            assert np.float32(twice.best_value) == np.float32(one.best_value)
            assert twice.n_evals == 2 * one.n_evals and twice.n_tie_evals == 2 * one.n_tie_evals
        # a result asked for in the middle of a sweep does not disturb it
        bsse.bsse_sweep_reset(g)
        bsse.bsse_sweep_chunk(g, X[:30000], 30000, 0)
        part = bsse.bsse_sweep_result(g)
        assert part.best_index < 30000
        bsse.bsse_sweep_chunk(g, X[30000:], count - 30000, 30000)
        _same(bsse.bsse_sweep_result(g), one)
        # an abandoned sweep leaves nothing behind
        bsse.bsse_sweep_reset(g)
        bsse.bsse_sweep_chunk(g, X[:777], 777, 10 ** 9)
        bsse.bsse_sweep_reset(g)
        bsse.bsse_sweep_chunk(g, X, count, 0)
        _same(bsse.bsse_sweep_result(g), one)


@pytest.mark.parametrize("shape", [(8, 8, 4), (8, 8, 12), (5, 7, 3), (32, 32, 16)])
def test_random_chunkings_in_random_order(shape):
    """Seeded random cuts of one batch, submitted in a random order, buffered and generated chunks
    mixed, some sweeps abandoned: every completed sweep gives the one-shot result."""
    import torch
    m, n, K = shape
    game = workloads.small_game(m, n, K, seed=70 + K, kind="normal")
    count = 30011
    rng = np.random.Generator(np.random.PCG64(123 + K))
    with _make(game) as g:
        X = torch.empty((count, m), dtype=torch.float32, device="cuda")
        bsse.bsse_dirichlet(g, 41, 0, count, X)
        one = bsse.bsse_sweep(g, X, count)
        for trial in range(12):
            ncuts = int(rng.integers(1, 9))
            cuts = np.unique(np.concatenate([[0, count], rng.integers(1, count, size=ncuts)]))
            spans = list(zip(cuts[:-1].tolist(), cuts[1:].tolist()))
            rng.shuffle(spans)
            bsse.bsse_sweep_reset(g)
            for lo, hi in spans:
                if rng.integers(0, 2):
                    bsse.bsse_sweep_dirichlet_chunk(g, 41, lo, hi - lo, lo)
                else:
                    bsse.bsse_sweep_chunk(g, X[lo:hi], hi - lo, lo)
            if trial % 4 == 3:
                continue                                     # abandoned: the next reset starts afresh
            _same(bsse.bsse_sweep_result(g), one)
            assert np.array_equal(bsse.bsse_sweep_best_row(g), X[one.best_index].cpu().numpy())


def test_streamed_sweep_on_a_stream_of_the_callers():
    """The handle bound to a stream of the caller's (default priority), a buffer filled on that stream
    between the chunks, two handles interleaved: generated chunks may run on the handles' own
    streams, and every result still equals the one-shot sweep."""
    import torch
    game_a = workloads.game(2)
    game_b = workloads.small_game(8, 8, 8, seed=5, kind="normal")
    count = 1 << 18
    side = torch.cuda.Stream()
    with _make(game_a) as ga, _make(game_b) as gb:
        ref_a = bsse.bsse_sweep_dirichlet(ga, 9, 0, 4 * count)
        ref_b = bsse.bsse_sweep_dirichlet(gb, 9, 0, 4 * count)
        bsse.bsse_set_stream(ga, side.cuda_stream)
        bsse.bsse_set_stream(gb, side.cuda_stream)
        X = torch.empty((count, 8), dtype=torch.float32, device="cuda")
        for rounds in range(3):
            bsse.bsse_sweep_reset(ga)
            bsse.bsse_sweep_reset(gb)
            with torch.cuda.stream(side):
                for k in range(4):
                    bsse.bsse_sweep_dirichlet_chunk(ga, 9, k * count, count, k * count)
                    if k == 2:
                        # a buffered chunk in the middle: rows written on the caller's stream just before
                        bsse.bsse_dirichlet(gb, 9, k * count, count, X)
                        bsse.bsse_sweep_chunk(gb, X, count, k * count)
                    else:
                        bsse.bsse_sweep_dirichlet_chunk(gb, 9, k * count, count, k * count)
                _same(bsse.bsse_sweep_result(ga), ref_a)
                _same(bsse.bsse_sweep_result(gb), ref_b)
        bsse.bsse_set_stream(ga, 0)
        bsse.bsse_set_stream(gb, 0)
        _same(bsse.bsse_sweep_dirichlet(ga, 9, 0, 4 * count), ref_a)
    torch.cuda.synchronize()


@pytest.mark.parametrize("cfg,count", [(2, 200000), (1, 30000)])
def test_against_the_oracle_on_its_own_rows(cfg, count):
    game = workloads.game(cfg)
    seed, first = 77, 1234
    Xo = odir.rows(seed, first, count, game.m).astype(np.float32)
    ref = osweep.sweep(game.A, game.B, game.prior, Xo, nthreads=8)
    with _make(game) as g:
        out = bsse.bsse_sweep_dirichlet(g, seed, first, count)
    assert out.n_evals == count * game.K
    v_ref, sc = osweep.value_under_profile(game.A, game.prior, Xo[out.best_index].astype(np.float64),
                                           out.best_response)
    # the device's rows differ from the oracle's by fp32 rounding of the generator (a few ulp)
    assert abs(out.best_value - v_ref) <= 2 * parity.TOL_F32 * max(sc, 1e-30)
    assert ref.values[out.best_index] >= ref.best_value - 2 * parity.TOL_F32 * max(sc, 1e-30)
    if out.best_index == ref.best_index:
        assert np.array_equal(out.best_response, ref.best_br)


def test_config2_at_bench_size_streamed_against_the_oracle():
    """The launch configuration bench.py times: config 2, chunks of 2^20 rows generated inside the
    sweep kernel, streamed (three chunks here), one result at the end.  The oracle generates and
    sweeps the same 3 * 2^20 rows itself."""
    game = workloads.game(2)
    count, chunks = 1 << 20, 3
    seed = game.candidate_seed
    Xo = odir.rows(seed, 0, chunks * count, game.m).astype(np.float32)
    ref = osweep.sweep(game.A, game.B, game.prior, Xo, nthreads=8)
    with _make(game) as g:
        bsse.bsse_sweep_reset(g)
        for k in range(chunks):
            bsse.bsse_sweep_dirichlet_chunk(g, seed, k * count, count, k * count)
        out = bsse.bsse_sweep_result(g)
        row = bsse.bsse_sweep_best_row(g)
    assert out.n_evals == chunks * count * game.K
    # the row the handle reports is the generator's row at the winning index (fp32 rounding apart)
    assert np.allclose(row, Xo[out.best_index], rtol=4e-6, atol=1e-9)
    v_ref, sc = osweep.value_under_profile(game.A, game.prior, Xo[out.best_index].astype(np.float64),
                                           out.best_response)
    assert abs(out.best_value - v_ref) <= 2 * parity.TOL_F32 * max(sc, 1e-30)
    assert ref.values[out.best_index] >= ref.best_value - 2 * parity.TOL_F32 * max(sc, 1e-30)
    assert out.best_index == ref.best_index            # the top two values are far apart here
    assert np.array_equal(out.best_response, ref.best_br)


def test_arguments():
    game = workloads.game(2)
    with _make(game) as g:
        out = bsse.bsse_sweep_dirichlet(g, 1, 0, 0)
        assert out.best_index == -1 and out.n_evals == 0
        with pytest.raises(bsse.BsseError) as e:
            bsse.bsse_sweep_best_row(g)
        assert e.value.status == bsse.BSSE_ESTATE
        for first, count in [(-1, 10), (0, -1)]:
            with pytest.raises(bsse.BsseError) as e:
                bsse.bsse_sweep_dirichlet(g, 1, first, count)
            assert e.value.status == bsse.BSSE_EINVAL
        with pytest.raises(bsse.BsseError) as e:
            bsse.bsse_sweep_dirichlet(g, 1, 0, (1 << 31) + 1)
        assert e.value.status == bsse.BSSE_EOVERFLOW
        with pytest.raises(bsse.BsseError) as e:
            bsse.bsse_sweep_dirichlet(g, 1, (1 << 63) - 5, 10)
        assert e.value.status == bsse.BSSE_EOVERFLOW
