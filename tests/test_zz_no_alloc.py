"""GPU test of bsse_sweep_static, the entry point that allocates nothing: its results against
bsse_sweep's on the same rows, call after call on the shared static scratch."""
import numpy as np
import pytest

from paper_2605_18856_amd import bsse, workloads

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def _make(game, path=bsse.BSSE_PATH_AUTO):
    storage = bsse.BSSE_STORAGE_BF16 if game.storage == "bf16" else bsse.BSSE_STORAGE_F32
    return bsse.bsse_create(game.m, game.n, game.K, game.A, game.B, game.prior, storage=storage, path=path)


def _same(a, b):
    assert (a.best_index, a.n_evals, a.n_tie_evals) == (b.best_index, b.n_evals, b.n_tie_evals)
    assert np.float64(a.best_value) == np.float64(b.best_value)
    if a.best_response is None:
        assert b.best_response is None
    else:
        assert np.array_equal(a.best_response, b.best_response)


# (m, n, K, payoff kind, storage, expected path prefix)
GAMES = [
    (3, 3, 2, "normal", "f32", "valu"),
    (8, 8, 4, "normal", "f32", "mfma_small_split6"),            # small-game kernel: running-best slots
    (8, 8, 16, "dup", "f32", "mfma_small_split6"),
    (32, 32, 16, "normal", "f32", "mfma_split6"),
    (64, 128, 4, "uniform", "bf16", "mfma_bf16"),
    (128, 256, 2, "int", "f32", "mfma_split3"),
    (6, 10, 3, "dup", "f32", "valu"),
]


@pytest.mark.parametrize("shape", GAMES, ids=lambda s: "m%dn%dK%d%s%s" % s[:5])
def test_static_sweep_equals_the_allocating_sweep(shape):
    """Two calls in a row, the second on a smaller input (the scratch still holds the first call's
    records), then a third on a larger one; every result equals bsse_sweep's bit for bit."""
    torch = _torch()
    m, n, K, kind, storage, prefix = shape
    game = workloads.small_game(m, n, K, 300 + m + n + K, kind=kind, storage=storage)
    cand = "dyadic" if kind == "dup" else "dirichlet"
    with _make(game) as g:
        assert bsse.bsse_path_name(g).startswith(prefix)
        for count in (40000 + 17, 1300, 1, 70001):
            X = workloads.host_candidates(m, count, 21 + count, cand)
            # put the best row late in the first call and early in the second: the winner moves
            Xd = torch.from_numpy(X).cuda()
            ref = bsse.bsse_sweep(g, Xd, count)
            got = bsse.bsse_sweep_static(g, Xd, count)
            _same(got, ref)
            again = bsse.bsse_sweep_static(g, Xd, count)
            _same(again, ref)
        if kind == "dup":
            assert ref.n_tie_evals > 0


def test_static_sweep_shared_by_two_handles_and_leaves_the_handle_usable():
    torch = _torch()
    ga = workloads.small_game(32, 32, 5, 71, kind="normal")
    gb = workloads.small_game(8, 8, 8, 72, kind="normal")
    Xa = torch.from_numpy(workloads.host_candidates(32, 5000, 73, "dirichlet")).cuda()
    Xb = torch.from_numpy(workloads.host_candidates(8, 3000, 74, "dirichlet")).cuda()
    with _make(ga) as a, _make(gb) as b:
        ra, rb = bsse.bsse_sweep(a, Xa, 5000), bsse.bsse_sweep(b, Xb, 3000)
        for _ in range(3):                       # the array holds the other handle's records each time
            _same(bsse.bsse_sweep_static(a, Xa, 5000), ra)
            _same(bsse.bsse_sweep_static(b, Xb, 3000), rb)
        # a smaller prefix through both entry points
        _same(bsse.bsse_sweep_static(a, Xa, 777), bsse.bsse_sweep(a, Xa, 777))
        # the static sweep is no result to polish, and does not disturb the handle's own sweeps
        bsse.bsse_sweep_static(a, Xa, 5000)
        with pytest.raises(bsse.BsseError) as e:
            bsse.bsse_polish(a)
        assert e.value.status == bsse.BSSE_ESTATE
        bsse.bsse_sweep_reset(a)
        bsse.bsse_sweep_chunk(a, Xa[:2500], 2500, 0)
        _same(bsse.bsse_sweep_static(b, Xb, 3000), rb)
        bsse.bsse_sweep_reset(a)
        bsse.bsse_sweep_chunk(a, Xa[:2500], 2500, 0)
        bsse.bsse_sweep_chunk(a, Xa[2500:], 2500, 2500)
        _same(bsse.bsse_sweep_result(a), ra)
        # empty input
        out = bsse.bsse_sweep_static(a, Xa, 0)
        assert out.best_index == -1 and out.best_response is None and out.n_evals == 0


def test_static_sweep_allocates_no_device_memory_and_rejects_what_exceeds_the_scratch():
    torch = _torch()
    game = workloads.small_game(3, 3, 2, 75, kind="normal")
    count = (1 << 22) + 64                       # one workgroup record more than the scratch holds
    X = torch.from_numpy(workloads.host_candidates(3, 4096, 76, "dirichlet")).cuda().repeat(count // 4096 + 1, 1)[:count].contiguous()
    with _make(game) as g:
        with pytest.raises(bsse.BsseError) as e:
            bsse.bsse_sweep_static(g, X, count)
        assert e.value.status == bsse.BSSE_EOVERFLOW
        ref = bsse.bsse_sweep(g, X, 1 << 22)
        torch.cuda.synchronize()
        free0 = torch.cuda.mem_get_info()[0]
        got = bsse.bsse_sweep_static(g, X, 1 << 22)      # exactly the maximum
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free0
        _same(got, ref)
        with pytest.raises(bsse.BsseError) as e:
            bsse.bsse_sweep_static(g, None, 0)
        assert e.value.status == bsse.BSSE_EINVAL
    # a fresh handle whose first call ever is the static one (nothing of its own scratch has been used)
    with _make(game) as h:
        free0 = torch.cuda.mem_get_info()[0]
        got = bsse.bsse_sweep_static(h, X, 50000)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free0
        _same(got, bsse.bsse_sweep(h, X, 50000))
