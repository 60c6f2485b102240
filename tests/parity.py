"""Comparison rules between the GPU library and the CPU oracle (used by the gpu tests,
smoke() and nothing in the product).

Best responses must agree exactly except where the oracle's own follower-payoff gap between
its best and second-best action is below 1e-6 of the dot-product scale s (flagged), or below
the worst-case fp32 accumulation bound 2*m*2^-24*s (bound-explained); anything else is a hard
failure.  Values are compared under the GPU's own best-response profile wherever that
profile differs, relative to sum_t p_t sum_i |x_i A_t[i][j_t]|.
"""
from dataclasses import dataclass

import numpy as np

from oracle import sweep as osweep
from paper_2605_18856_amd import workloads

TOL_F32 = 1e-5
TOL_BF16 = 2e-3


@dataclass
class ParityReport:
    n_evals: int
    br_mismatch: int
    flagged: int
    bound_explained: int
    hard_failures: int
    max_value_err: float      # max |V_gpu - V_oracle| / scale over candidates
    value_failures: int


def oracle_inputs(game, X):
    """The operand values the kernel is defined to consume, for the oracle."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    if game.storage == "bf16":
        return (workloads.round_to_bf16(game.A), workloads.round_to_bf16(game.B),
                workloads.round_to_bf16(X))
    return game.A, game.B, X


def compare_eval(game, X, V_gpu, br_gpu, tol=None, nthreads=8) -> ParityReport:
    tol = tol if tol is not None else (TOL_BF16 if game.storage == "bf16" else TOL_F32)
    A, B, Xo = oracle_inputs(game, X)
    ref = osweep.sweep(A, B, game.prior, Xo, diagnostics=True, nthreads=nthreads)
    C, K = br_gpu.shape
    m = game.m
    mism = br_gpu != ref.br
    flagged = mism & (ref.gap < 1e-6 * ref.scale)
    bound = mism & ~flagged & (ref.gap < 2.0 * m * 2.0 ** -24 * ref.scale)
    hard = mism & ~flagged & ~bound
    # values: oracle value under the GPU's profile where it differs
    V_ref = ref.values.copy()
    A64 = np.asarray(A, np.float64)
    p64 = np.asarray(game.prior, np.float64)
    Xo64 = Xo.astype(np.float64)
    # scale for every candidate: sum_t p_t sum_i |x_i A_t[i, j_t]|
    scale = np.zeros(C)
    absX = np.abs(Xo64)
    for t in range(K):
        cols = np.abs(A64[t])[:, br_gpu[:, t].astype(np.int64)]          # [m][C]
        scale += p64[t] * np.einsum("ci,ic->c", absX, cols)
    for c in np.nonzero(mism.any(axis=1))[0]:
        V_ref[c], scale[c] = osweep.value_under_profile(A, game.prior, Xo64[c], br_gpu[c])
    err = np.abs(V_gpu.astype(np.float64) - V_ref) / np.maximum(scale, 1e-30)
    return ParityReport(C * K, int(mism.sum()), int(flagged.sum()), int(bound.sum()),
                        int(hard.sum()), float(err.max()) if C else 0.0, int((err > tol).sum()))


def check_report(rep: ParityReport, tol):
    assert rep.hard_failures == 0, rep
    assert rep.value_failures == 0 and rep.max_value_err <= tol, rep
    # tolerated mismatches must stay rare
    assert rep.flagged + rep.bound_explained <= max(2, rep.n_evals // 1000), rep


def check_winner(game, X, outcome, V_gpu, tol=None):
    """The sweep's winner against the oracle's, and against a CPU arg-max over the GPU's own
    per-candidate values (bit-exact: greatest value, lowest index)."""
    tol = tol if tol is not None else (TOL_BF16 if game.storage == "bf16" else TOL_F32)
    c_cpu = int(np.argmax(V_gpu))                      # numpy returns the first maximum
    assert outcome.best_index == c_cpu
    assert np.float32(outcome.best_value) == V_gpu[c_cpu]
    A, B, Xo = oracle_inputs(game, X)
    ref = osweep.sweep(A, B, game.prior, Xo, nthreads=8)
    _, sc = osweep.value_under_profile(A, game.prior, Xo[outcome.best_index].astype(np.float64),
                                       ref.br[outcome.best_index])
    assert ref.values[outcome.best_index] >= ref.best_value - tol * max(sc, 1e-30)
    return outcome.best_index == ref.best_index
