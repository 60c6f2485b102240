/* Host-sanitizer driver for the CPU oracle (test infrastructure): built with
 * -fsanitize=address,undefined by tests/test_sanitizers.py and run on the CPU.  It walks the
 * oracle's entry points over the shapes the tests use (hand game, ragged counts, zero
 * candidates, float and double rows, one and several threads, optional outputs present and
 * absent) and checks a few fixed results, so that a memory or arithmetic error in the oracle
 * itself cannot hide behind the values it is used to judge. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double bsse_oracle_value_under_profile(int m, int n, int K, const double *A, const double *prior,
                                       const double *x, const int32_t *br, double *abs_scale);
int bsse_oracle_sweep(int m, int n, int K, const double *A, const double *B, const double *prior,
                      const void *X, int x_is_f32, int64_t C, double *V_out, int32_t *br_out,
                      double *gap_out, double *scale_out, double *best_value, int64_t *best_index,
                      int32_t *best_br, int nthreads);

static int failures = 0;
#define CHECK(c)                                                                      \
    do {                                                                              \
        if (!(c)) { fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #c); ++failures; } \
    } while (0)

static uint64_t lcg_state = 0x9E3779B97F4A7C15ull;
static double lcg(void)
{
    lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(lcg_state >> 11) / 9007199254740992.0;
}

static void hand_game(void)
{
    /* Leader payoffs [[2,4],[1,3]], follower payoffs the identity, one type: at x = (1/2, 1/2) both
     * columns are best responses and the leader-favourable one (column 1) gives 3.5. */
    const double A[4] = { 2, 4, 1, 3 }, B[4] = { 1, 0, 0, 1 }, p[1] = { 1.0 };
    const double X[6] = { 1.0, 0.0, 0.5, 0.5, 0.25, 0.75 };
    double V[3], gap[3], sc[3], bv;
    int32_t br[3], bbr[1];
    int64_t bi;
    const int used = bsse_oracle_sweep(2, 2, 1, A, B, p, X, 0, 3, V, br, gap, sc, &bv, &bi, bbr, 1);
    CHECK(used == 1);
    CHECK(V[0] == 2.0 && br[0] == 0);
    CHECK(V[1] == 3.5 && br[1] == 1 && gap[1] == 0.0);
    CHECK(V[2] == 3.25 && br[2] == 1);
    CHECK(bi == 1 && bv == 3.5 && bbr[0] == 1);
    double s = -1.0;
    const int32_t prof[1] = { 1 };
    CHECK(bsse_oracle_value_under_profile(2, 2, 1, A, p, X + 2, prof, &s) == 3.5 && s == 3.5);
    CHECK(bsse_oracle_value_under_profile(2, 2, 1, A, p, X + 2, prof, NULL) == 3.5);
}

static void random_game(int m, int n, int K, int64_t C)
{
    double *A = malloc(sizeof(double) * (size_t)K * m * n), *B = malloc(sizeof(double) * (size_t)K * m * n);
    double *p = malloc(sizeof(double) * (size_t)K);
    double *Xd = malloc(sizeof(double) * (size_t)(C > 0 ? C : 1) * m);
    float *Xf = malloc(sizeof(float) * (size_t)(C > 0 ? C : 1) * m);
    double psum = 0.0;
    for (int i = 0; i < K * m * n; ++i) { A[i] = 2.0 * lcg() - 1.0; B[i] = floor(8.0 * lcg()) - 4.0; }
    for (int t = 0; t < K; ++t) { p[t] = lcg() + 0.1; psum += p[t]; }
    for (int t = 0; t < K; ++t) p[t] /= psum;
    for (int64_t c = 0; c < C; ++c) {
        double s = 0.0;
        for (int i = 0; i < m; ++i) { Xd[c * m + i] = -log(lcg() + 1e-300); s += Xd[c * m + i]; }
        for (int i = 0; i < m; ++i) { Xd[c * m + i] /= s; Xf[c * m + i] = (float)Xd[c * m + i]; }
    }
    double *V1 = malloc(sizeof(double) * (size_t)(C > 0 ? C : 1)), *V4 = malloc(sizeof(double) * (size_t)(C > 0 ? C : 1));
    int32_t *br1 = malloc(sizeof(int32_t) * (size_t)(C > 0 ? C : 1) * K), *br4 = malloc(sizeof(int32_t) * (size_t)(C > 0 ? C : 1) * K);
    double *gap = malloc(sizeof(double) * (size_t)(C > 0 ? C : 1) * K), *sc = malloc(sizeof(double) * (size_t)(C > 0 ? C : 1) * K);
    int32_t *bb1 = malloc(sizeof(int32_t) * (size_t)K), *bb4 = malloc(sizeof(int32_t) * (size_t)K);
    double bv1 = 0, bv4 = 0;
    int64_t bi1 = -2, bi4 = -2;
    CHECK(bsse_oracle_sweep(m, n, K, A, B, p, Xd, 0, C, V1, br1, gap, sc, &bv1, &bi1, bb1, 1) == 1);
    const int used = bsse_oracle_sweep(m, n, K, A, B, p, Xd, 0, C, V4, br4, NULL, NULL, &bv4, &bi4, bb4, 4);
    CHECK(used >= 1);
    CHECK(bi1 == bi4);
    if (C == 0) {
        CHECK(bi1 == -1);
    } else {
        CHECK(bv1 == bv4 && memcmp(bb1, bb4, sizeof(int32_t) * (size_t)K) == 0);
        CHECK(memcmp(V1, V4, sizeof(double) * (size_t)C) == 0);
        CHECK(memcmp(br1, br4, sizeof(int32_t) * (size_t)C * K) == 0);
        for (int64_t c = 0; c < C; ++c) {
            double s;
            const double v = bsse_oracle_value_under_profile(m, n, K, A, p, Xd + c * m, br1 + c * K, &s);
            CHECK(fabs(v - V1[c]) <= 1e-12 * (s > 1.0 ? s : 1.0));
            CHECK(V1[c] <= bv1);
            for (int t = 0; t < K; ++t) CHECK(br1[c * K + t] >= 0 && br1[c * K + t] < n && gap[c * K + t] >= 0.0 && sc[c * K + t] >= 0.0);
        }
        CHECK(V1[bi1] == bv1);
        /* float rows, no optional outputs at all */
        double bvf = 0;
        int64_t bif = -2;
        CHECK(bsse_oracle_sweep(m, n, K, A, B, p, Xf, 1, C, NULL, NULL, NULL, NULL, &bvf, &bif, bb4, 3) >= 1);
        CHECK(bif >= 0 && bif < C && fabs(bvf - bv1) <= 1e-5 * (fabs(bv1) + 1.0));
    }
    free(A); free(B); free(p); free(Xd); free(Xf); free(V1); free(V4); free(br1); free(br4); free(gap); free(sc);
    free(bb1); free(bb4);
}

int main(void)
{
    hand_game();
    random_game(5, 7, 3, 1000);
    random_game(1, 1, 1, 5);
    random_game(8, 8, 4, 257);
    random_game(3, 130, 2, 33);
    random_game(4, 4, 2, 0);
    if (failures) { fprintf(stderr, "%d check(s) failed\n", failures); return 1; }
    puts("oracle sanitizer driver: ok");
    return 0;
}
