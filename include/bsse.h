/*
 * bsse.h -- C ABI of libbsse: the batched commitment sweep of a finite Bayesian
 * Stackelberg game on one AMD MI355X (gfx950).
 *
 * Subject.  The paper this library is named after gives no formula, algorithm or
 * example for the subject (it only names it, in its preamble); every operation below
 * is therefore defined by the textbook strong Stackelberg equilibrium of a finite
 * Bayesian game, restated here:
 *
 *   A leader (the overseer) has m actions, a follower (the model) has n actions and
 *   one of K types t with prior weight prior[t].  A_t[i][j] is the leader's payoff
 *   and B_t[i][j] the type-t follower's payoff when the leader plays i and the
 *   follower plays j.  The leader commits to a mixed strategy x (a candidate row of
 *   m numbers).  A type-t follower answers with
 *       j*_t(x) = the action maximising  u_t[j] = sum_i x[i]*B_t[i][j];
 *                 among maximisers, one maximising  l_t[j] = sum_i x[i]*A_t[i][j];
 *                 among those, the lowest j           (strong-Stackelberg tie-break)
 *   and the leader's value of x is  V(x) = sum_t prior[t] * l_t[j*_t(x)].
 *   The sweep evaluates V on every candidate and returns the greatest value, the
 *   lowest candidate index attaining it, and that candidate's K best responses.
 *
 * Arithmetic.  Payoffs are held in fp32 (or bf16, on request) and every sum is
 * accumulated in fp32; "maximiser" and "equal" mean exact equality of the fp32
 * numbers the kernel itself computed.  The summation order inside a dot product is
 * an implementation detail (MFMA paths do not sum in index order; the split path
 * forms each product from bf16 parts, see bsse_options.path).
 *
 * Conventions.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP device
 *     memory on the game's device (e.g. torch.Tensor.data_ptr()).
 *   - Matrices A and B are host, row-major [K][m][n]; they are copied and repacked at
 *     create and the caller keeps ownership.  Candidates are device, row-major
 *     [count][m] fp32 (4-byte aligned; 16-byte aligned when m is a multiple of 4, so that
 *     any row of an aligned buffer qualifies), borrowed for the duration of the call (until
 *     the stream has run the enqueued work, for the asynchronous calls).  Rows are NOT checked to lie on
 *     the simplex: the sweep is defined for any finite x.  Non-finite candidates give
 *     an unspecified result (never a fault).
 *   - Every function returns a bsse_status.  Arguments are validated before any HIP
 *     call, so argument errors are reported on a machine without a GPU.  On error no
 *     output argument is written.  bsse_last_error() gives a thread-local message.
 *   - A game handle is not thread-safe; distinct handles are independent.  All device
 *     work of a handle is enqueued on its stream (default: the null stream).
 *   - The library never falls back to the CPU: without a usable gfx950 device every
 *     call that needs one returns BSSE_EDEVICE.
 */
#ifndef BSSE_H
#define BSSE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bsse_game bsse_game; /* opaque: packed payoffs, workspace, running best */

typedef enum {
    BSSE_OK = 0,
    BSSE_EINVAL = 1,     /* bad dimension, null pointer, bad option, prior off the simplex */
    BSSE_ENOTFINITE = 2, /* a payoff or prior entry is NaN or infinite */
    BSSE_EOVERFLOW = 3,  /* a count does not fit (lattice size, buffer size) */
    BSSE_ENOMEM = 4,     /* host or device allocation failed */
    BSSE_EDEVICE = 5,    /* no usable device, or a HIP call failed */
    BSSE_ESTATE = 6      /* call out of order (e.g. sweep of generated candidates before generating) */
} bsse_status;

enum { BSSE_STORAGE_F32 = 0, BSSE_STORAGE_BF16 = 1 };
enum { BSSE_PATH_AUTO = 0, BSSE_PATH_VALU = 1, BSSE_PATH_MFMA = 2, BSSE_PATH_MFMA_SPLIT = 3 };

typedef struct {
    int storage; /* BSSE_STORAGE_*: how payoffs (and, for BF16, candidates) enter the
                    contraction.  BF16 rounds payoffs and each candidate component to
                    bfloat16 (nearest, ties to even) and accumulates in fp32. */
    int path;    /* BSSE_PATH_*.  MFMA = matrix cores in the storage type (fp32 MFMA for F32,
                    bf16 MFMA for BF16).  MFMA_SPLIT (F32 storage only) = bf16 matrix cores on
                    fp32 operands: every payoff and candidate component is split into bf16
                    parts hi + mid + lo (exactly, up to the last part's rounding) and the
                    products hi*hi, hi*mid, mid*hi, hi*lo, mid*mid, lo*hi are accumulated in
                    fp32 (three products when every payoff is itself a bf16 number); the
                    omitted products are below 2^-24 of the terms, so the result is within
                    fp32 rounding of the fp32 dot product.  AUTO picks, in this order, the
                    small-game kernel, MFMA_SPLIT, MFMA, VALU, by what the shape supports.
                    Games with m = n = 8 and K in {4, 8, 12, 16} (fp32 storage) run on the
                    small-game kernel under AUTO and MFMA alike: bf16 matrix cores on split
                    operands as under MFMA_SPLIT, at fp32 accuracy (bsse_path_name says
                    "mfma_small_split6").  A forced path on an unsupported shape is BSSE_EINVAL. */
    int device;  /* HIP device ordinal; -1 = the calling thread's current device */
} bsse_options;

typedef struct {
    double  best_value;   /* V of the winning candidate (the kernel's fp32 value, widened) */
    int64_t best_index;   /* its index in the swept sequence (index_base + row); -1 if none */
    int64_t n_evals;      /* candidate-type evaluations accumulated since the last reset */
    int64_t n_tie_evals;  /* of those, evaluations where two or more follower actions tied
                             exactly for the maximum (diagnostic) */
} bsse_result;

/* Problem statement (see top).  m, n, K >= 1; A, B: host [K][m][n]; prior: host [K],
 * finite, >= 0, |sum - 1| <= 1e-6 (checked, not renormalised).  Limits: m <= 4096,
 * n <= 65535, K <= 65535, K*m*n <= 2^28.  bsse_create = bsse_create_ex with
 * {BSSE_STORAGE_F32, BSSE_PATH_AUTO, -1}.  *out is owned by the caller: bsse_destroy. */
bsse_status bsse_create(int m, int n, int K, const float *A, const float *B,
                        const float *prior, bsse_game **out);
bsse_status bsse_create_ex(int m, int n, int K, const float *A, const float *B,
                           const float *prior, const bsse_options *opt, bsse_game **out);
void bsse_destroy(bsse_game *g); /* NULL is allowed */

/* Stream (a hipStream_t passed as void*; NULL = null stream) on which all later work
 * of this handle is enqueued.  The caller keeps the stream alive. */
bsse_status bsse_set_stream(bsse_game *g, void *hip_stream);

/* Candidate generation, step 1 of the sweep.
 *
 * bsse_lattice: generates on the device every point of the simplex lattice of
 * resolution N (N >= 1): x = k/N for the compositions k of N into m non-negative
 * parts, in ascending lexicographic order of (k_0..k_{m-1}); each component is
 * fl32(k_i)/fl32(N), correctly rounded.  The buffer belongs to the handle and replaces
 * any earlier generated set; *count_out = C(N+m-1, m-1).  BSSE_EOVERFLOW if that count
 * exceeds 2^40 or the buffer cannot be allocated within device memory.
 *
 * bsse_lattice_count: the same count, host only (no device needed).
 *
 * bsse_dirichlet: rows first..first+count-1 of the seeded sequence of points uniform
 * on the simplex (flat Dirichlet): component i of row c is g_i * fl32(1 / sum_i g_i) with
 * g_i = -ln(u_i), u_i = ((w_i >> 8) + 1) / 2^24, and w the output words of
 * Philox4x32-10 keyed by (seed low word, seed high word) at counter
 * (c low word, c high word, i / 4, 0), word i % 4.  Row c depends on (seed, c) only -- not on
 * first, count, or the alignment of out_dev.
 * out_dev = device [count][m] fp32 written by the call (asynchronously on the
 * handle's stream), or NULL to write a handle-owned buffer that replaces any earlier
 * generated set. */
bsse_status bsse_lattice(bsse_game *g, int N, int64_t *count_out);
bsse_status bsse_lattice_count(int m, int N, int64_t *count_out);
bsse_status bsse_dirichlet(bsse_game *g, uint64_t seed, int64_t first, int64_t count,
                           float *out_dev);

/* Local sets for refinement around a survivor of a sweep: the same generators with every point t
 * replaced by the convex combination (1 - radius) * centre + radius * t, i.e. the simplex (and
 * the set on it) shrunk by `radius` towards `centre`; component i is computed as
 * fl32(fl32(radius * t_i) + fl32(fl32(1 - radius) * centre[i])) (three separately rounded fp32
 * operations).  centre = host [m], finite (a point of the simplex keeps the set on the simplex;
 * not checked); 0 <= radius <= 1 (1 = the plain set, 0 = the centre repeated).  Otherwise as
 * bsse_lattice / bsse_dirichlet. */
bsse_status bsse_lattice_around(bsse_game *g, int N, const float *centre, float radius,
                                int64_t *count_out);
bsse_status bsse_dirichlet_around(bsse_game *g, uint64_t seed, int64_t first, int64_t count,
                                  const float *centre, float radius, float *out_dev);

/* The handle-owned generated set: *dev_out = device pointer ([*count_out][m] fp32),
 * valid until the next generation call or destroy.  BSSE_ESTATE if none. */
bsse_status bsse_candidates(bsse_game *g, const float **dev_out, int64_t *count_out);

/* The sweep, steps 2-5 (follower payoffs, tie-broken best responses, leader value,
 * arg-max over candidates), in one call: resets the running best, sweeps `count` rows
 * of `candidates_dev` (NULL = the handle-owned generated set, count must then equal
 * its size or be 0 meaning "all"), waits for the stream, and fills *res and
 * best_response_out (host, K int32, may be NULL).  count == 0 with explicit candidates
 * is allowed: best_index = -1 and best_response_out is untouched. */
bsse_status bsse_sweep(bsse_game *g, const float *candidates_dev, int64_t count,
                       bsse_result *res, int32_t *best_response_out);

/* bsse_sweep for callers that cannot allocate: code that must not call hipMalloc (tight serving
 * loops, harnesses that forbid allocation, code that will later be captured into a HIP graph).
 * Same arguments, same result bit for bit as bsse_sweep on the same rows, but every piece of device
 * scratch (workgroup records, running best, winning row, tie counter, running-best slots) lives in
 * a static device array of 1.2 MiB that each GPU the library runs on holds until the process ends;
 * the call performs no hipMalloc / hipHostMalloc / hipFree and creates no stream or event.
 * candidates_dev must be given (not NULL).  Limits: the chunk may need at most 65536 workgroup
 * records (2^24 candidates on the matrix-core paths with 256 candidates per workgroup, 2^22 on
 * the plain vector path; the small-game kernel has no such limit); more is BSSE_EOVERFLOW, with
 * nothing enqueued.  All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (two handles, two streams, two threads) race on it and must be serialised by the
 * caller.  Kernel timing (bsse_set_timing) does not cover this call.  Like bsse_sweep it resets
 * the handle's streamed sweep; afterwards there is no result to polish (bsse_polish: BSSE_ESTATE). */
bsse_status bsse_sweep_static(bsse_game *g, const float *candidates_dev, int64_t count,
                              bsse_result *res, int32_t *best_response_out);

/* The same sweep streamed in chunks (step 6, the running best over chunks):
 *   bsse_sweep_reset  forgets the running best;
 *   bsse_sweep_chunk  enqueues the sweep of one chunk whose row r has global index
 *                     index_base + r, and merges its best into the running best: greater
 *                     value, then lower global index, so the result is that of one sweep
 *                     over all chunks in index order, whatever order they are submitted
 *                     in; it does not wait for the device; the winning row is copied into
 *                     the handle, so the chunk buffer may be reused once the stream has
 *                     passed it;
 *   bsse_sweep_result waits for the stream and reports like bsse_sweep. */
bsse_status bsse_sweep_reset(bsse_game *g);
bsse_status bsse_sweep_chunk(bsse_game *g, const float *candidates_dev, int64_t count,
                             int64_t index_base);
bsse_status bsse_sweep_result(bsse_game *g, bsse_result *res, int32_t *best_response_out);

/* The row of the running best (the candidate at best_index of the sweep so far), copied from the
 * handle: x_out = host [m] fp32.  Waits for the stream.  BSSE_ESTATE if no candidate has been
 * swept since the last reset. */
bsse_status bsse_sweep_best_row(bsse_game *g, float *x_out);

/* Steps 1-6 without a candidate buffer: the sweep of rows first..first+count-1 of the seeded
 * flat-Dirichlet sequence (exactly the rows bsse_dirichlet(g, seed, first, count, X) writes; the
 * result is, bit for bit, that of bsse_sweep(g, X, count, ...): row first + r has index r).  For
 * games that run the small-game kernel (m = n = 8, K in {4, 8, 12, 16}, fp32) the rows are produced
 * in registers inside the sweep kernel and never reach memory; for every other game they pass
 * through a staging buffer of the handle (at most 2^26 floats), piece by piece.  The winning
 * row itself is bsse_sweep_best_row, or bsse_dirichlet(g, seed, first + best_index, 1, out).
 *   bsse_sweep_dirichlet        resets, sweeps, waits and reports like bsse_sweep;
 *   bsse_sweep_dirichlet_chunk  the streamed form, like bsse_sweep_chunk (row first + r has global
 *                               index index_base + r); report with bsse_sweep_result.
 * Chunks of generated rows read nothing the caller's stream produces, so the handle may run them
 * on streams of its own (default priority), ordered behind the work enqueued on the handle's
 * stream before them; the next bsse_sweep_result / bsse_sweep_best_row / bsse_sweep_reset + chunk
 * makes the handle's stream wait for them.  Work the caller enqueues on its stream in between is
 * therefore not ordered after such chunks until one of those calls.
 * first, count >= 0, count <= 2^31; BSSE_EOVERFLOW if first + count or index_base + count
 * overflows. */
bsse_status bsse_sweep_dirichlet(bsse_game *g, uint64_t seed, int64_t first, int64_t count,
                                 bsse_result *res, int32_t *best_response_out);
bsse_status bsse_sweep_dirichlet_chunk(bsse_game *g, uint64_t seed, int64_t first, int64_t count,
                                       int64_t index_base);

/* Per-candidate outputs of the same kernels (steps 2-4 without the arg-max), for
 * checking: values_dev_out = device [count] fp32, br_dev_out = device [count][K] int32;
 * either may be NULL.  Enqueued on the handle's stream; does not wait. */
bsse_status bsse_eval(bsse_game *g, const float *candidates_dev, int64_t count,
                      float *values_dev_out, int32_t *br_dev_out);

/* Prior-robustness batch: the sweep of bsse_sweep for P priors over the same game and the same
 * candidates in one pass.  A follower's best response does not depend on the prior, so the
 * contraction and the best responses are computed once and every prior costs K multiply-adds per
 * candidate.  priors = host [P][K], each row checked like bsse_create's prior; 1 <= P <= 65536.
 * res = host [P]; best_response_out = host [P][K] int32 or NULL.  For prior p the result is the
 * greatest V_p(x_c) = sum_t priors[p][t] * l_t[j*_t(x_c)] (fp32 fused multiply-adds, t
 * ascending), the lowest candidate index attaining it, and that candidate's best responses; the
 * handle's own prior plays no part.  The value is the same fp32 number as a sweep of a handle
 * created with that prior would give whenever that sweep sums its types in the same order (all
 * paths but the small-game kernel, which adds two half sums).  n_tie_evals is the same for every
 * prior.  Waits for the stream; its scratch (up to 1 GiB for the leader payoffs of a chunk of
 * candidates, plus the records) is allocated on first use, grown when a later call needs more,
 * and kept until bsse_destroy; does not touch the running best of the streamed sweep. */
bsse_status bsse_sweep_priors(bsse_game *g, const float *candidates_dev, int64_t count,
                              const float *priors, int P, bsse_result *res,
                              int32_t *best_response_out);

/* Top-k: the k best candidates of the sweep instead of the best one, in the order "greater V
 * first, lower index among equal values" (so entry 0 is bsse_sweep's answer).  1 <= k <= 256.
 * values_out = host [k] (the kernels' fp32 values, widened), indices_out = host [k],
 * best_response_out = host [k][K] int32 or NULL; *found_out = min(k, count) entries are written.
 * The handle's prior is used.  Waits for the stream; its scratch (4 bytes per candidate of a
 * chunk of at most 2^26, plus records) is allocated on first use, grown when a later call needs
 * more, and kept until bsse_destroy; does not touch the running best of the streamed sweep. */
bsse_status bsse_sweep_topk(bsse_game *g, const float *candidates_dev, int64_t count, int k,
                            double *values_out, int64_t *indices_out, int32_t *best_response_out,
                            int *found_out);

/* Refinement: top-k and local re-sweeps in rounds, starting from the handle-owned generated set
 * (BSSE_ESTATE if none).  The k best candidates of that set are the first centres; in every
 * round a local set is generated around each centre -- the lattice of resolution lattice_N
 * (bsse_lattice_around) when lattice_N > 0, else cloud_count Dirichlet rows
 * (bsse_dirichlet_around with seed + round * 1000003 + centre number) -- and swept with
 * bsse_sweep_topk; the k best distinct points among the centres and everything found become the
 * next centres, and the radius is multiplied by shrink.  1 <= k <= 256, 1 <= rounds <= 64,
 * radius and shrink in (0, 1]; exactly one of lattice_N, cloud_count positive.  x_out = host [m]
 * the best point found, res->best_value its V as the kernels compute it (never below the best of
 * the starting set), res->best_index = -1, res->n_evals the evaluations spent,
 * best_response_out = host [K] or NULL.  The handle-owned set is overwritten.  Waits for the
 * stream. */
bsse_status bsse_refine(bsse_game *g, int k, int rounds, int lattice_N, int64_t cloud_count,
                        uint64_t seed, float radius, float shrink, float *x_out, bsse_result *res,
                        int32_t *best_response_out);

/* LP polish.  The sweep only sees its candidates; the linear program of the winner's best-response
 * profile lands on the exact vertex of that profile's region (one program of the multiple-LPs
 * characterisation of the strong Stackelberg equilibrium):
 *     maximise   sum_t prior[t] * x . A_t[:, j_t]
 *     subject to x . (B_t[:, j_t] - B_t[:, j']) >= 0  for every t and j' != j_t,  x on the simplex.
 *
 * bsse_profile_lp: host only, no device needed.  Solves that program in fp64 (simplex method on
 * the dual, whose tableau has m rows) for the game given by host arrays laid out as for
 * bsse_create (prior: finite, >= 0; its sum is not checked) and profile = host [K] actions.
 * *feasible_out = 1 and x_out (host [m], on the simplex), *value_out filled; or *feasible_out = 0
 * when the profile is a best response to no x (x_out, value_out untouched).  BSSE_EOVERFLOW when
 * m * (2 + K(n-1) + m) exceeds 2^28, BSSE_ESTATE if the method does not converge.
 *
 * bsse_polish: polishes the result of the last completed sweep of the handle: the one
 * bsse_sweep / bsse_sweep_dirichlet / bsse_sweep_result last reported, with no chunk or reset
 * since (BSSE_ESTATE otherwise).  profile = host [K], or NULL for the winner's own best responses.  Solves the program
 * with the payoffs as given to create (fp32, also for BF16 storage), then evaluates, with the
 * sweep's own kernels, eight points of the segment from the program's vertex to the sweep's
 * winner (the vertex lies on the boundary of the profile's region, where rounding x to fp32 can
 * tip a follower over to another action; V is linear along the segment inside the region) and
 * keeps the best: x_out (host [m] fp32), res->best_value = its V as the kernels compute it,
 * res->best_index = which point (0 = the vertex ... 7 = the sweep's winner), best_response_out
 * (host [K], may be NULL) its best responses, *lp_value_out (may be NULL) the program's optimum.
 * Then  V(sweep's winner) <= res->best_value <= equilibrium value, and *lp_value_out is the most
 * any commitment with that profile can earn (the equilibrium value itself when the profile is
 * the equilibrium's).  BSSE_EINVAL if the given profile is a best response nowhere.  Waits for
 * the stream. */
/* bsse_solve_realised: the multiple-LPs solve restricted to the follower profiles the sweep
 * realises.  Evaluates the candidates (bsse_eval's outputs), collects the distinct best-response
 * profiles, and solves the program of each, most promising first (by the best swept value under
 * the profile), at most max_profiles of them.  *value_out = the greatest program optimum, x_out =
 * host [m] its vertex (fp32), profile_out = host [K] its profile (may be NULL),
 * *n_profiles_out = distinct profiles realised, *n_solved_out = programs solved.  Every program
 * optimum is attainable (at the vertex, by the leader-favourable tie-break), so
 *     best swept value <= *value_out <= equilibrium value,
 * with equality on the right whenever the equilibrium's profile is among those solved -- then
 * this is the exact strong Stackelberg equilibrium for n_solved programs instead of n^K.
 * count * K <= 2^27.  Waits for the stream. */
bsse_status bsse_solve_realised(bsse_game *g, const float *candidates_dev, int64_t count,
                                int max_profiles, float *x_out, double *value_out,
                                int32_t *profile_out, int *n_profiles_out, int *n_solved_out);
bsse_status bsse_profile_lp(int m, int n, int K, const float *A, const float *B, const float *prior,
                            const int32_t *profile, double *x_out, double *value_out,
                            int *feasible_out);
bsse_status bsse_polish(bsse_game *g, const int32_t *profile, float *x_out, bsse_result *res,
                        int32_t *best_response_out, double *lp_value_out);

/* Which kernel family the handle uses: "valu", "mfma_f32", "mfma_bf16", "mfma_split3",
 * "mfma_split6", ... (static string). */
const char *bsse_path_name(const bsse_game *g);

/* Kernel timing for roofline reports.  When enabled, every launch of the fused sweep
 * kernel (payoffs + best response + value + block arg-max) is bracketed by HIP events on
 * the handle's stream; bsse_get_timing waits for the stream and returns the summed
 * duration in milliseconds and the number of launches since timing was enabled. */
bsse_status bsse_set_timing(bsse_game *g, int enabled);
bsse_status bsse_get_timing(bsse_game *g, double *kernel_ms_out, int64_t *launches_out);

/* Measured ceilings of the device (diagnostics for roofline reports; no part of the sweep): what
 * plain kernels reach on it, to be quoted beside the vendor peaks.  *stream_read_gbs: a streaming
 * read of a 2 GiB buffer, GB/s; *mfma_bf16_tflops, *mfma_f32_tflops: a loop of independent
 * 32x32x16 bf16 / 32x32x2 fp32 matrix-core instructions on every compute unit, TFLOP/s;
 * *empty_launch_us: time per launch of 2000 empty kernels enqueued back to back.  device = HIP
 * ordinal, -1 = current.  Allocates 2 GiB for the duration of the call; uses the null stream and
 * waits for it.  All four outputs are host pointers and must not be NULL. */
bsse_status bsse_measure_ceilings(int device, double *stream_read_gbs, double *mfma_bf16_tflops,
                                  double *mfma_f32_tflops, double *empty_launch_us);

/* One more measured ceiling (diagnostics; no part of the sweep): the rate the bf16 matrix cores
 * keep, in TFLOP/s of 32x32x16 instructions, when every wavefront alternates blocks of
 * mfma_per_round matrix instructions (a multiple of 4, at most 4096) with blocks of valu_per_round
 * independent vector instructions (a multiple of 24, at most 65536: three-operand maxima, compares
 * into scalar masks and selects under them in equal parts), two wavefronts per SIMD on every
 * compute unit, nothing loaded or stored.  With the counts of a sweep kernel's instruction mix it
 * says what that mix could reach without loads, dependencies and barriers.  device = HIP ordinal,
 * -1 = current; uses the null stream and waits for it; the output is a host pointer. */
bsse_status bsse_measure_mixed_ceiling(int device, int mfma_per_round, int valu_per_round,
                                       double *mfma_bf16_tflops);

const char *bsse_last_error(void); /* thread-local; "" if none */
const char *bsse_status_name(bsse_status s);

#ifdef __cplusplus
}
#endif
#endif /* BSSE_H */
