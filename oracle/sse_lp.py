"""Exact strong Stackelberg equilibrium of a small Bayesian game by the multiple-LPs
method.  TEST INFRASTRUCTURE ONLY; it pins the sweep oracle, nothing else uses it.

For every pure follower profile (j_1..j_K), one per type, solve

    maximise   sum_t p_t * x . A_t[:, j_t]
    subject to x . (B_t[:, j_t] - B_t[:, j']) >= 0   for every type t and action j'
               x in the simplex

(the profile is a best response to x exactly on that polytope).  The equilibrium value is
the best optimum over feasible profiles, n^K linear programs in all.  Because the
follower breaks ties in the leader's favour, V(x) equals the maximum, over the profiles
that are best responses at x, of the profile's objective; hence V(x) <= V_LP for every x,
with equality at an optimiser.  The LPs are solved by scipy's HiGHS ``linprog``.
"""
from itertools import product

import numpy as np
from scipy.optimize import linprog


def solve(A, B, prior):
    """Returns (value, x, profile) of the strong Stackelberg equilibrium."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    p = np.asarray(prior, dtype=np.float64)
    K, m, n = A.shape
    best = (-np.inf, None, None)
    for prof in product(range(n), repeat=K):
        c = np.zeros(m)
        rows = []
        for t, j in enumerate(prof):
            c -= p[t] * A[t][:, j]                       # linprog minimises
            for jp in range(n):
                if jp != j:
                    rows.append(B[t][:, jp] - B[t][:, j])   # <= 0
        A_ub = np.asarray(rows) if rows else None
        b_ub = np.zeros(len(rows)) if rows else None
        res = linprog(c, A_ub=A_ub, b_ub=b_ub, A_eq=np.ones((1, m)), b_eq=[1.0],
                      bounds=[(0, None)] * m, method="highs")
        if res.status == 0 and -res.fun > best[0]:
            best = (-res.fun, res.x.copy(), tuple(prof))
    return best


def profile_lp(A, B, prior, profile):
    """The linear program of ONE follower profile: (feasible, value, x).  Same program as one
    pass of the loop in ``solve`` (kept apart so that a single profile can be checked)."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    p = np.asarray(prior, dtype=np.float64)
    K, m, n = A.shape
    c = np.zeros(m)
    rows = []
    for t, j in enumerate(profile):
        c -= p[t] * A[t][:, j]
        for jp in range(n):
            if jp != j:
                rows.append(B[t][:, jp] - B[t][:, j])
    A_ub = np.asarray(rows) if rows else None
    b_ub = np.zeros(len(rows)) if rows else None
    res = linprog(c, A_ub=A_ub, b_ub=b_ub, A_eq=np.ones((1, m)), b_eq=[1.0],
                  bounds=[(0, None)] * m, method="highs")
    if res.status != 0:
        return False, None, None
    return True, -res.fun, res.x.copy()


def maximin(A):
    """Value and strategy of the row player's maximin LP for matrix A (m x n):
    max v s.t. x.A[:, j] >= v for all j, x in the simplex."""
    A = np.asarray(A, dtype=np.float64)
    m, n = A.shape
    c = np.zeros(m + 1)
    c[-1] = -1.0
    A_ub = np.hstack([-A.T, np.ones((n, 1))])
    res = linprog(c, A_ub=A_ub, b_ub=np.zeros(n),
                  A_eq=np.hstack([np.ones((1, m)), np.zeros((1, 1))]), b_eq=[1.0],
                  bounds=[(0, None)] * m + [(None, None)], method="highs")
    assert res.status == 0
    return -res.fun, res.x[:m]
