/*
 * bsse_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain fp64 CPU statement of the commitment sweep of a finite Bayesian
 * Stackelberg game.  It exists to check the GPU library and to be timed beside
 * it; the product never calls it.  It shares no code with the GPU path.
 *
 * The paper this repository is named after only names the subject (in its
 * preamble) and states no formula for it.  What is computed here is therefore the textbook
 * definition of the strong Stackelberg equilibrium of a finite Bayesian game,
 * evaluated by brute force over a given candidate list:
 *
 *   leader commits to a mixed strategy x in R^m (a candidate row);
 *   a follower of type t (prior weight p_t) sees x and plays a pure action j
 *   maximising its expected payoff  u_t[j] = sum_i x[i] * B_t[i][j];
 *   among its maximisers it plays one that is best for the leader, i.e. that
 *   maximises  l_t[j] = sum_i x[i] * A_t[i][j]; among those, the lowest j;
 *   the leader's value of x is  V(x) = sum_t p_t * l_t[j*_t];
 *   the sweep returns the candidate of greatest V, lowest index among equals.
 *
 * Every sum runs in ascending index order in fp64; "equal" is exact fp64
 * equality.  No blocking, no reordering, no tolerance.
 *
 * Layout: A and B are [K][m][n] row-major (type, leader action, follower
 * action); candidates are [C][m] row-major.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* One candidate x (m doubles).  Writes K best responses to br (may not be
 * NULL), and, when non-NULL, per-type diagnostics:
 *   gap[t]   = (largest follower payoff) - (second largest follower payoff),
 *              counting equal payoffs at different j as gap 0; +inf when n==1
 *   scale[t] = max over those two actions of sum_i |x[i] * B_t[i][j]|
 * Returns V(x). */
static double eval_candidate(int m, int n, int K, const double *A, const double *B,
                             const double *prior, const double *x, int32_t *br,
                             double *gap, double *scale)
{
    double V = 0.0;
    for (int t = 0; t < K; ++t) {
        const double *Bt = B + (size_t)t * m * n;
        const double *At = A + (size_t)t * m * n;

        /* follower payoffs: first pass finds the maximum and the runner-up */
        double umax = -INFINITY, usecond = -INFINITY;
        int jmax = -1, jsecond = -1;
        for (int j = 0; j < n; ++j) {
            double u = 0.0;
            for (int i = 0; i < m; ++i) u += x[i] * Bt[(size_t)i * n + j];
            if (u > umax) { usecond = umax; jsecond = jmax; umax = u; jmax = j; }
            else if (u > usecond) { usecond = u; jsecond = j; }
        }

        /* second pass: among exact maximisers, best for the leader, then lowest j */
        int jstar = -1;
        double lstar = -INFINITY;
        for (int j = 0; j < n; ++j) {
            double u = 0.0;
            for (int i = 0; i < m; ++i) u += x[i] * Bt[(size_t)i * n + j];
            if (u != umax) continue;
            double l = 0.0;
            for (int i = 0; i < m; ++i) l += x[i] * At[(size_t)i * n + j];
            if (jstar < 0 || l > lstar) { jstar = j; lstar = l; }
        }
        br[t] = jstar;
        V += prior[t] * lstar;

        if (gap) gap[t] = (jsecond < 0) ? INFINITY : (umax - usecond);
        if (scale) {
            double s = 0.0;
            int js[2] = { jmax, jsecond };
            for (int q = 0; q < 2; ++q) {
                if (js[q] < 0) continue;
                double a = 0.0;
                for (int i = 0; i < m; ++i) a += fabs(x[i] * Bt[(size_t)i * n + js[q]]);
                if (a > s) s = a;
            }
            scale[t] = s;
        }
    }
    return V;
}

/* Leader value of candidate x when the followers are told to play the given
 * profile br[K] (no best-response step): sum_t p_t * sum_i x[i]*A_t[i][br[t]].
 * Also returns, through *abs_scale when non-NULL, sum_t p_t*sum_i|x[i]*A_t[i][br[t]]|. */
double bsse_oracle_value_under_profile(int m, int n, int K, const double *A,
                                       const double *prior, const double *x,
                                       const int32_t *br, double *abs_scale)
{
    double V = 0.0, S = 0.0;
    for (int t = 0; t < K; ++t) {
        const double *At = A + (size_t)t * m * n;
        double l = 0.0, a = 0.0;
        for (int i = 0; i < m; ++i) {
            double term = x[i] * At[(size_t)i * n + br[t]];
            l += term;
            a += fabs(term);
        }
        V += prior[t] * l;
        S += prior[t] * a;
    }
    if (abs_scale) *abs_scale = S;
    return V;
}

/*
 * Sweep C candidates.  X is [C][m]; x_is_f32 != 0 means X points to float
 * (each value is widened to double, nothing else), otherwise to double.
 * Optional per-candidate outputs (NULL to skip): V_out[C], br_out[C*K],
 * gap_out[C*K], scale_out[C*K].  Always written: *best_value, *best_index,
 * best_br[K] (best_index = -1 and nothing else written when C == 0).
 * nthreads <= 1 runs the loop sequentially; otherwise candidates are split
 * over that many OpenMP threads (each candidate is still evaluated by the
 * sequential routine above, and the final arg-max is taken sequentially).
 * Returns the number of threads actually used, or -1 on allocation failure.
 */
int bsse_oracle_sweep(int m, int n, int K, const double *A, const double *B,
                      const double *prior, const void *X, int x_is_f32, int64_t C,
                      double *V_out, int32_t *br_out, double *gap_out, double *scale_out,
                      double *best_value, int64_t *best_index, int32_t *best_br,
                      int nthreads)
{
    int used = 1;
    *best_index = -1;
    if (C <= 0) return used;

    double *Vbuf = V_out ? V_out : (double *)malloc((size_t)C * sizeof(double));
    if (!Vbuf) return -1;
    int failed = 0;

#ifdef _OPENMP
    if (nthreads > 1) used = nthreads;
#pragma omp parallel num_threads(used)
#endif
    {
        double *xrow = (double *)malloc((size_t)m * sizeof(double));
        int32_t *brrow = (int32_t *)malloc((size_t)K * sizeof(int32_t));
        if (!xrow || !brrow) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp barrier
#endif
        if (!failed) {
#ifdef _OPENMP
#pragma omp for schedule(static)
#endif
            for (int64_t c = 0; c < C; ++c) {
                if (x_is_f32) {
                    const float *xf = (const float *)X + (size_t)c * m;
                    for (int i = 0; i < m; ++i) xrow[i] = (double)xf[i];
                } else {
                    memcpy(xrow, (const double *)X + (size_t)c * m, (size_t)m * sizeof(double));
                }
                int32_t *brp = br_out ? br_out + (size_t)c * K : brrow;
                Vbuf[c] = eval_candidate(m, n, K, A, B, prior, xrow, brp,
                                         gap_out ? gap_out + (size_t)c * K : NULL,
                                         scale_out ? scale_out + (size_t)c * K : NULL);
            }
        }
        free(xrow);
        free(brrow);
    }
    if (failed) { if (!V_out) free(Vbuf); return -1; }

    /* arg-max over candidates: greatest value, lowest index among equals */
    int64_t cstar = 0;
    for (int64_t c = 1; c < C; ++c)
        if (Vbuf[c] > Vbuf[cstar]) cstar = c;
    *best_value = Vbuf[cstar];
    *best_index = cstar;

    /* best responses of the winner (re-evaluated; deterministic) */
    {
        double *xrow = (double *)malloc((size_t)m * sizeof(double));
        if (!xrow) { if (!V_out) free(Vbuf); return -1; }
        if (x_is_f32) {
            const float *xf = (const float *)X + (size_t)cstar * m;
            for (int i = 0; i < m; ++i) xrow[i] = (double)xf[i];
        } else {
            memcpy(xrow, (const double *)X + (size_t)cstar * m, (size_t)m * sizeof(double));
        }
        (void)eval_candidate(m, n, K, A, B, prior, xrow, best_br, NULL, NULL);
        free(xrow);
    }
    if (!V_out) free(Vbuf);
    return used;
}
