// The linear program of one pure follower profile (host code, no device work).
//
// For a profile j = (j_t), one follower action per type, the leader's best commitment among
// those to which j is a best response is
//     maximise   c . x,   c_i = sum_t p_t A_t[i][j_t]
//     subject to x . (B_t[:, j_t] - B_t[:, j']) >= 0   for every type t and action j' != j_t,
//                sum_i x_i = 1,  x >= 0
// (one program of the classical multiple-LPs characterisation of the strong Stackelberg
// equilibrium).  It has m variables and R = K(n-1) constraints, so its dual
//     minimise   lambda   subject to   lambda - (G^T y)_i - s_i = c_i,   y >= 0, s >= 0
// (G the R x m matrix of payoff differences) has only m rows; that is the one solved here, by
// the tableau simplex method in fp64.  The dual is always feasible (y = 0, lambda = max c), so
// there is no first phase: subtracting the row of the largest c_i from the others gives a
// starting basis {lambda, s_i (i != k)} with a non-negative right-hand side.  An unbounded dual
// means the profile is a best response nowhere on the simplex.  At the optimum the primal
// solution x is read off the reduced costs of the slack columns s_i.
#include "bsse_internal.h"
#include <cmath>
#include <vector>

namespace bsse {

int solve_profile_lp(int m, int n, int K, const float *A, const float *B, const float *prior,
                     const int32_t *profile, double *x_out, double *value_out)
{
    const int R = K * (n - 1);
    const int ncol = 2 + R + m;                  // lambda+, lambda-, y_r, s_i
    const int col_y = 2, col_s = 2 + R;
    std::vector<double> c((size_t)m, 0.0);
    for (int t = 0; t < K; ++t)
        for (int i = 0; i < m; ++i)
            c[i] += (double)prior[t] * (double)A[((size_t)t * m + i) * n + profile[t]];
    double cmin = c[0];
    for (int i = 1; i < m; ++i) cmin = c[i] < cmin ? c[i] : cmin;
    const double shift = 1.0 - cmin;             // c + shift >= 1; the optimum moves by the same amount
    int k = 0;
    for (int i = 1; i < m; ++i) if (c[i] > c[k]) k = i;

    // tableau rows (m of them), right-hand side apart
    std::vector<double> T((size_t)m * ncol, 0.0), rhs((size_t)m), d((size_t)ncol, 0.0);
    std::vector<int> basic((size_t)m);
    double scale = 1.0;
    for (int i = 0; i < m; ++i) {
        double *row = &T[(size_t)i * ncol];
        row[0] = 1.0; row[1] = -1.0;
        int r = 0;
        for (int t = 0; t < K; ++t) {
            const float *Bt = B + (size_t)t * m * n + (size_t)i * n;
            const double bj = (double)Bt[profile[t]];
            for (int j = 0; j < n; ++j) {
                if (j == profile[t]) continue;
                const double gri = bj - (double)Bt[j];
                row[col_y + r] = -gri;
                scale = std::fabs(gri) > scale ? std::fabs(gri) : scale;
                ++r;
            }
        }
        row[col_s + i] = -1.0;
        rhs[i] = c[i] + shift;
    }
    for (int i = 0; i < m; ++i) {
        if (i == k) continue;
        double *row = &T[(size_t)i * ncol];
        const double *rk = &T[(size_t)k * ncol];
        for (int j = 0; j < ncol; ++j) row[j] = rk[j] - row[j];
        rhs[i] = rhs[k] - rhs[i];
        basic[i] = col_s + i;
    }
    basic[k] = 0;
    // reduced costs of "minimise lambda+ - lambda-": only row k holds a basic variable with a cost
    for (int j = 0; j < ncol; ++j) d[j] = (j == 0 ? 1.0 : j == 1 ? -1.0 : 0.0) - T[(size_t)k * ncol + j];
    double z = rhs[k];

    const double tol = 1e-11 * scale;
    const long long max_iter = 200LL * (m + R) + 1000;
    int stall = 0;
    for (long long it = 0; it < max_iter; ++it) {
        // entering column: most negative reduced cost; lowest index while the objective stalls
        // (degenerate pivots), which cannot cycle
        int e = -1;
        if (stall < 40) {
            double best = -tol;
            for (int j = 0; j < ncol; ++j) if (d[j] < best) { best = d[j]; e = j; }
        } else {
            for (int j = 0; j < ncol; ++j) if (d[j] < -tol) { e = j; break; }
        }
        if (e < 0) {                              // optimal
            double s = 0.0;
            for (int i = 0; i < m; ++i) { double v = d[col_s + i]; v = v > 0.0 ? v : 0.0; x_out[i] = v; s += v; }
            if (!(s > 0.0)) return 2;
            for (int i = 0; i < m; ++i) x_out[i] /= s;
            *value_out = z - shift;
            return 0;
        }
        // leaving row: least ratio; among (near-)equal ratios the lowest basic variable
        int l = -1;
        double best_ratio = 0.0;
        for (int i = 0; i < m; ++i) {
            const double a = T[(size_t)i * ncol + e];
            if (a <= tol) continue;
            const double ratio = rhs[i] / a;
            if (l < 0 || ratio < best_ratio - 1e-13 * (1.0 + std::fabs(best_ratio)) ||
                (ratio <= best_ratio + 1e-13 * (1.0 + std::fabs(best_ratio)) && basic[i] < basic[l])) {
                l = i; best_ratio = ratio;
            }
        }
        if (l < 0) return 1;                      // dual unbounded: the profile is nowhere a best response
        // pivot on (l, e)
        double *rl = &T[(size_t)l * ncol];
        const double piv = rl[e];
        for (int j = 0; j < ncol; ++j) rl[j] /= piv;
        rhs[l] /= piv;
        rl[e] = 1.0;
        for (int i = 0; i < m; ++i) {
            if (i == l) continue;
            double *ri = &T[(size_t)i * ncol];
            const double f = ri[e];
            if (f == 0.0) continue;
            for (int j = 0; j < ncol; ++j) ri[j] -= f * rl[j];
            ri[e] = 0.0;
            rhs[i] -= f * rhs[l];
            if (rhs[i] < 0.0 && rhs[i] > -1e-9 * (1.0 + std::fabs(rhs[l]))) rhs[i] = 0.0;
        }
        const double f = d[e];
        for (int j = 0; j < ncol; ++j) d[j] -= f * rl[j];
        d[e] = 0.0;
        const double z_new = z + f * rhs[l];
        stall = (z - z_new > 1e-14 * (1.0 + std::fabs(z))) ? 0 : stall + 1;
        z = z_new;
        basic[l] = e;
    }
    return 2;                                     // iteration limit
}

}  // namespace bsse
