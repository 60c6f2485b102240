// Host-sanitizer driver for the library's host code (test infrastructure): linked against the
// library's sources compiled with -fsanitize=address,undefined on the host side by
// tests/test_sanitizers.py and run on the CPU, with or without a GPU in the machine.  It walks
// the C ABI's argument checks (which come before any device call), the host-only entry points
// (lattice count, status names, the profile linear program) and, when no device is present, the
// clean failure of handle creation after the host packing has run.
#include "../../include/bsse.h"
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

static int failures = 0;
#define CHECK(c)                                                                      \
    do {                                                                              \
        if (!(c)) { std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #c); ++failures; } \
    } while (0)

static uint64_t lcg_state = 0x2545F4914F6CDD1Dull;
static double lcg()
{
    lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(lcg_state >> 11) / 9007199254740992.0;
}

static void status_names()
{
    for (int s = 0; s <= 6; ++s) CHECK(bsse_status_name((bsse_status)s) && bsse_status_name((bsse_status)s)[0]);
    CHECK(bsse_status_name((bsse_status)99) != nullptr);
    CHECK(bsse_last_error() != nullptr);
}

static void lattice_counts()
{
    int64_t c = -1;
    CHECK(bsse_lattice_count(3, 100, &c) == BSSE_OK && c == 5151);
    CHECK(bsse_lattice_count(1, 7, &c) == BSSE_OK && c == 1);
    CHECK(bsse_lattice_count(8, 1, &c) == BSSE_OK && c == 8);
    CHECK(bsse_lattice_count(0, 4, &c) == BSSE_EINVAL);
    CHECK(bsse_lattice_count(3, 0, &c) == BSSE_EINVAL);
    CHECK(bsse_lattice_count(3, 4, nullptr) == BSSE_EINVAL);
    CHECK(bsse_lattice_count(64, 1000000, &c) == BSSE_EOVERFLOW);
}

static void create_errors()
{
    const int m = 3, n = 3, K = 2;
    std::vector<float> A(K * m * n), B(K * m * n);
    for (size_t i = 0; i < A.size(); ++i) { A[i] = (float)i; B[i] = (float)(A.size() - i); }
    const float p[2] = { 0.7f, 0.3f };
    bsse_options opt = { BSSE_STORAGE_F32, BSSE_PATH_AUTO, -1 };
    bsse_game *h = nullptr;
    const int bad[][3] = { { 0, 3, 2 }, { 3, 0, 2 }, { 3, 3, 0 }, { -1, 3, 2 }, { 5000, 3, 2 }, { 3, 70000, 2 } };
    for (auto &d : bad) {
        CHECK(bsse_create_ex(d[0], d[1], d[2], A.data(), B.data(), p, &opt, &h) == BSSE_EINVAL && h == nullptr);
        CHECK(bsse_last_error()[0] != 0);
    }
    CHECK(bsse_create_ex(m, n, K, nullptr, B.data(), p, &opt, &h) == BSSE_EINVAL);
    CHECK(bsse_create_ex(m, n, K, A.data(), nullptr, p, &opt, &h) == BSSE_EINVAL);
    CHECK(bsse_create_ex(m, n, K, A.data(), B.data(), nullptr, &opt, &h) == BSSE_EINVAL);
    CHECK(bsse_create_ex(m, n, K, A.data(), B.data(), p, nullptr, &h) == BSSE_EINVAL);
    CHECK(bsse_create_ex(m, n, K, A.data(), B.data(), p, &opt, nullptr) == BSSE_EINVAL);
    bsse_options o2 = opt;
    o2.storage = 7;
    CHECK(bsse_create_ex(m, n, K, A.data(), B.data(), p, &o2, &h) == BSSE_EINVAL);
    o2 = opt; o2.path = 9;
    CHECK(bsse_create_ex(m, n, K, A.data(), B.data(), p, &o2, &h) == BSSE_EINVAL);
    const float pbad[2] = { 0.7f, 0.7f };
    CHECK(bsse_create_ex(m, n, K, A.data(), B.data(), pbad, &opt, &h) == BSSE_EINVAL);
    std::vector<float> An = A;
    An[4] = NAN;
    CHECK(bsse_create_ex(m, n, K, An.data(), B.data(), p, &opt, &h) == BSSE_ENOTFINITE);
    CHECK(h == nullptr);
    // Valid arguments: with a device this makes a handle, without one it must fail cleanly after
    // the host-side work; both shapes of game packing (small-game kernel and general) are tried.
    const bsse_status st = bsse_create_ex(m, n, K, A.data(), B.data(), p, &opt, &h);
    CHECK(st == BSSE_OK || st == BSSE_EDEVICE || st == BSSE_ENOMEM);
    CHECK((st == BSSE_OK) == (h != nullptr));
    bsse_destroy(h);
    h = nullptr;
    std::vector<float> A8(4 * 8 * 8), B8(4 * 8 * 8);
    for (size_t i = 0; i < A8.size(); ++i) { A8[i] = (float)lcg(); B8[i] = (float)lcg(); }
    const float p4[4] = { 0.25f, 0.25f, 0.25f, 0.25f };
    const bsse_status st8 = bsse_create_ex(8, 8, 4, A8.data(), B8.data(), p4, &opt, &h);
    CHECK(st8 == BSSE_OK || st8 == BSSE_EDEVICE || st8 == BSSE_ENOMEM);
    bsse_destroy(h);
    bsse_destroy(nullptr);
}

static void null_handle_errors()
{
    int64_t c = 0;
    bsse_result r;
    float x[4] = { 0 };
    double d = 0;
    int i0 = 0, i1 = 0;
    int32_t br[4] = { 0 };
    const float *dev = nullptr;
    CHECK(bsse_set_stream(nullptr, nullptr) == BSSE_EINVAL);
    CHECK(bsse_lattice(nullptr, 4, &c) == BSSE_EINVAL);
    CHECK(bsse_dirichlet(nullptr, 1, 0, 4, nullptr) == BSSE_EINVAL);
    CHECK(bsse_lattice_around(nullptr, 4, x, 0.1f, &c) == BSSE_EINVAL);
    CHECK(bsse_dirichlet_around(nullptr, 1, 0, 4, x, 0.1f, nullptr) == BSSE_EINVAL);
    CHECK(bsse_candidates(nullptr, &dev, &c) == BSSE_EINVAL);
    CHECK(bsse_sweep(nullptr, nullptr, 0, &r, br) == BSSE_EINVAL);
    CHECK(bsse_sweep_static(nullptr, nullptr, 0, &r, br) == BSSE_EINVAL);
    CHECK(bsse_sweep_reset(nullptr) == BSSE_EINVAL);
    CHECK(bsse_sweep_chunk(nullptr, nullptr, 0, 0) == BSSE_EINVAL);
    CHECK(bsse_sweep_result(nullptr, &r, br) == BSSE_EINVAL);
    CHECK(bsse_sweep_best_row(nullptr, x) == BSSE_EINVAL);
    CHECK(bsse_sweep_dirichlet(nullptr, 1, 0, 4, &r, br) == BSSE_EINVAL);
    CHECK(bsse_sweep_dirichlet_chunk(nullptr, 1, 0, 4, 0) == BSSE_EINVAL);
    CHECK(bsse_eval(nullptr, nullptr, 0, nullptr, nullptr) == BSSE_EINVAL);
    CHECK(bsse_polish(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == BSSE_EINVAL);
    CHECK(bsse_solve_realised(nullptr, nullptr, 0, 1, x, &d, br, &i0, &i1) == BSSE_EINVAL);
    CHECK(bsse_set_timing(nullptr, 1) == BSSE_EINVAL);
    CHECK(bsse_get_timing(nullptr, &d, &c) == BSSE_EINVAL);
    CHECK(bsse_path_name(nullptr) != nullptr);
    CHECK(bsse_measure_ceilings(0, nullptr, &d, &d, &d) == BSSE_EINVAL);
    CHECK(bsse_measure_ceilings(-5, &d, &d, &d, &d) == BSSE_EINVAL);
}

// value of x under the profile and the largest violation of the best-response constraints
static void lp_check(int m, int n, int K, const std::vector<float> &A, const std::vector<float> &B,
                     const std::vector<float> &p, const std::vector<int32_t> &prof, const std::vector<double> &x,
                     double value)
{
    double sum = 0, obj = 0;
    for (int i = 0; i < m; ++i) { CHECK(x[i] >= -1e-12); sum += x[i]; }
    CHECK(std::fabs(sum - 1.0) <= 1e-9);
    for (int t = 0; t < K; ++t) {
        double l = 0;
        for (int i = 0; i < m; ++i) l += x[i] * A[((size_t)t * m + i) * n + prof[t]];
        obj += p[t] * l;
        double uj = 0, umax = -1e300;
        for (int j = 0; j < n; ++j) {
            double u = 0;
            for (int i = 0; i < m; ++i) u += x[i] * B[((size_t)t * m + i) * n + j];
            if (j == prof[t]) uj = u;
            if (u > umax) umax = u;
        }
        CHECK(uj >= umax - 1e-7 * (std::fabs(umax) + 1.0));
    }
    CHECK(std::fabs(obj - value) <= 1e-7 * (std::fabs(value) + 1.0));
}

static void profile_lps()
{
    {   // the hand game: optimum 3.5 at (1/2, 1/2) under column 1, 2 at (1, 0) under column 0
        const float A[4] = { 2, 4, 1, 3 }, B[4] = { 1, 0, 0, 1 }, p[1] = { 1.0f };
        double x[2], v = 0;
        int ok = -1;
        int32_t prof = 1;
        CHECK(bsse_profile_lp(2, 2, 1, A, B, p, &prof, x, &v, &ok) == BSSE_OK && ok == 1);
        CHECK(std::fabs(v - 3.5) < 1e-12 && std::fabs(x[0] - 0.5) < 1e-12 && std::fabs(x[1] - 0.5) < 1e-12);
        prof = 0;
        CHECK(bsse_profile_lp(2, 2, 1, A, B, p, &prof, x, &v, &ok) == BSSE_OK && ok == 1);
        CHECK(std::fabs(v - 2.0) < 1e-12 && std::fabs(x[0] - 1.0) < 1e-12);
        prof = 2;
        CHECK(bsse_profile_lp(2, 2, 1, A, B, p, &prof, x, &v, &ok) == BSSE_EINVAL);
        prof = 0;
        CHECK(bsse_profile_lp(2, 2, 1, nullptr, B, p, &prof, x, &v, &ok) == BSSE_EINVAL);
        CHECK(bsse_profile_lp(2, 2, 1, A, B, p, nullptr, x, &v, &ok) == BSSE_EINVAL);
        float Ainf[4] = { 2, INFINITY, 1, 3 };
        CHECK(bsse_profile_lp(2, 2, 1, Ainf, B, p, &prof, x, &v, &ok) == BSSE_ENOTFINITE);
    }
    const int shapes[][3] = { { 3, 3, 2 }, { 5, 4, 3 }, { 8, 8, 4 }, { 2, 9, 1 }, { 12, 5, 6 } };
    for (auto &sh : shapes) {
        const int m = sh[0], n = sh[1], K = sh[2];
        std::vector<float> A((size_t)K * m * n), B((size_t)K * m * n), p(K);
        for (auto &a : A) a = (float)(2.0 * lcg() - 1.0);
        for (auto &b : B) b = (float)(std::floor(6.0 * lcg()) - 3.0);       // integers: ties and degenerate vertices
        float ps = 0;
        for (auto &q : p) { q = (float)(lcg() + 0.05); ps += q; }
        for (auto &q : p) q /= ps;
        int feasible = 0;
        for (int rep = 0; rep < 40; ++rep) {
            std::vector<int32_t> prof(K);
            for (auto &j : prof) j = (int32_t)(lcg() * n) % n;
            std::vector<double> x(m, -1.0);
            double v = 0;
            int ok = -1;
            CHECK(bsse_profile_lp(m, n, K, A.data(), B.data(), p.data(), prof.data(), x.data(), &v, &ok) == BSSE_OK);
            CHECK(ok == 0 || ok == 1);
            if (ok == 1) { ++feasible; lp_check(m, n, K, A, B, p, prof, x, v); }
        }
        (void)feasible;
    }
}

int main()
{
    status_names();
    lattice_counts();
    create_errors();
    null_handle_errors();
    profile_lps();
    if (failures) { std::fprintf(stderr, "%d check(s) failed\n", failures); return 1; }
    std::puts("abi sanitizer driver: ok");
    return 0;
}
