"""Top-k reduction (bsse_sweep_topk): bit-exact against a CPU sort of the GPU's own per-candidate
values by (value descending, index ascending), and against the oracle at the survivors."""
import numpy as np
import pytest

from oracle import sweep as osweep
from paper_2605_18856_amd import bsse, workloads
from tests import parity
from tests.test_gpu_parity import _make, _run_eval

pytestmark = pytest.mark.gpu


def _expected(V, k):
    order = np.lexsort((np.arange(V.shape[0]), -V.astype(np.float64)))     # value desc, index asc
    return order[:k]


@pytest.mark.parametrize("shape,count,k", [((3, 3, 2), 50, 8), ((3, 3, 2), 5, 8), ((8, 8, 4), 8192, 16),
                                           ((8, 8, 4), 8193, 1), ((8, 8, 4), 100000, 64),
                                           ((5, 7, 3), 30000, 256), ((32, 32, 4), 20000, 10),
                                           ((64, 128, 2), 9000, 5)])
def test_topk_against_cpu_sort_and_oracle(shape, count, k):
    m, n, K = shape
    storage = "bf16" if m == 64 else "f32"
    game = workloads.small_game(m, n, K, seed=300 + m, kind="uniform" if storage == "bf16" else "normal",
                                storage=storage)
    tol = parity.TOL_BF16 if storage == "bf16" else parity.TOL_F32
    X = workloads.host_candidates(m, count, seed=21, kind="dirichlet")
    with _make(game) as g:
        Xd, V, br = _run_eval(g, X)
        vals, idx, brs = bsse.bsse_sweep_topk(g, k, Xd, count)
        top1 = bsse.bsse_sweep(g, Xd, count)
    exp = _expected(V, k)
    assert idx.shape[0] == min(k, count)
    assert np.array_equal(idx, exp)
    assert np.array_equal(vals.astype(np.float32), V[exp])
    assert np.array_equal(brs, br[exp])
    assert idx[0] == top1.best_index and np.float32(vals[0]) == np.float32(top1.best_value)
    # the survivors' values against the oracle (under the reported profiles)
    A, B, Xo = parity.oracle_inputs(game, X)
    for r in range(min(len(idx), 8)):
        v_ref, sc = osweep.value_under_profile(A, game.prior, Xo[idx[r]].astype(np.float64), brs[r])
        assert abs(vals[r] - v_ref) <= tol * max(sc, 1e-30)


def test_equal_values_keep_index_order():
    """Duplicated candidates have bit-identical values: the lower index comes first."""
    game = workloads.small_game(8, 8, 4, seed=2, kind="normal")
    base = workloads.host_candidates(8, 300, seed=3, kind="dirichlet")
    X = np.concatenate([base, base, base[:100]], axis=0)
    with _make(game) as g:
        Xd, V, br = _run_eval(g, X)
        vals, idx, _ = bsse.bsse_sweep_topk(g, 12, Xd, X.shape[0])
    assert np.array_equal(idx, _expected(V, 12))
    assert idx[1] == idx[0] + 300 and vals[0] == vals[1]          # first copy, then second copy


def test_more_than_one_chunk():
    """2^26 + 4097 candidates of the config-2 game: two value chunks, merged by a final level."""
    import torch
    game = workloads.game(2)
    count = (1 << 26) + 4097
    with _make(game) as g:
        Xd = torch.empty((count, game.m), dtype=torch.float32, device="cuda")
        bsse.bsse_dirichlet(g, 5, 0, count, Xd)
        # plant the best row of the first chunk again at the very end: equal value, higher index
        top = bsse.bsse_sweep(g, Xd, 1 << 26)
        Xd[count - 1] = Xd[top.best_index]
        vals, idx, brs = bsse.bsse_sweep_topk(g, 32, Xd, count)
        V = torch.empty(count, dtype=torch.float32, device="cuda")
        bsse.bsse_eval(g, Xd, count, V, None)
        torch.cuda.synchronize()
        # CPU check on the GPU's own values: top 32 by (value desc, index asc)
        Vh = V.cpu().numpy()
    cand = np.argpartition(-Vh, 4096)[:4096]
    cand = cand[np.lexsort((cand, -Vh[cand].astype(np.float64)))][:32]
    assert np.array_equal(idx, cand)
    assert np.array_equal(vals.astype(np.float32), Vh[cand])
    pos = list(idx)
    assert top.best_index in pos and count - 1 in pos
    assert pos.index(top.best_index) < pos.index(count - 1)


def test_argument_errors_and_empty():
    game = workloads.small_game(3, 3, 2, seed=1, kind="normal")
    X = workloads.host_candidates(3, 10, seed=1, kind="dirichlet")
    with _make(game) as g:
        Xd, _, _ = _run_eval(g, X)
        for k in (0, 257):
            with pytest.raises(bsse.BsseError) as e:
                bsse.bsse_sweep_topk(g, k, Xd, 10)
            assert e.value.status == bsse.BSSE_EINVAL
        vals, idx, brs = bsse.bsse_sweep_topk(g, 4, Xd, 0)
        assert len(vals) == 0 and len(idx) == 0
