// Internal declarations shared by the translation units of libbsse (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bsse {

// Device view of one game, passed to kernels by value.  All pointers are device memory
// owned by the handle.
struct GameView {
    int m, n, K;
    int x_bf16;           // 1: round each candidate component to bf16 before use
    const float *B;       // [K][m][n]  follower payoffs, row-major (VALU path)
    const float *AT;      // [K][n][m]  leader payoffs, one follower action's column contiguous
    const float *prior;   // [K]
    // MFMA paths (null when the shape has no MFMA packing)
    const void *Bpack;    // follower payoffs in MFMA A-operand fragment order
    const void *ATpack;   // leader payoffs [K][n][m_pad] in the contraction's k order
    int m_pad;            // m rounded up to the MFMA k granularity
    int n_pad;            // n rounded up to the row-tile granularity (see sweep_mfma.hip)
    int variant;          // matrix-core kernel variant chosen at create (see mfma_select)
};

// Running best over chunks, in device memory.
struct RunningBest {
    float value;
    int   has;               // 0 until a chunk has been merged
    long long index;
    unsigned long long ties; // tie evaluations of all merged chunks
};

// Small-game kernel, sweep mode.  Workgroup b keeps its own running best over the chunks of a
// sweep in slot b (read and rewritten by that workgroup alone, so chunk launches need no grid
// stage and no synchronisation); a one-workgroup kernel folds the slots when the result is asked
// for.  A slot belongs to the current sweep when its epoch matches.
struct SmallSlot {
    float value;
    unsigned epoch;
    long long index;         // global candidate index
    unsigned br[2];          // packed best responses (three bits per type; one word per lane half)
    unsigned pad[2];
    float x[8];              // the row itself
};

struct SmallSweep {
    SmallSlot *slots;        // [small_num_slots()]; nullptr outside the small-game sweep
    unsigned epoch;
};

// Fold of the slots into the result of the sweep.
struct FinishArgs {
    const SmallSlot *slots;
    int nslots;
    unsigned epoch;
    int first;               // != 0: first fold of this sweep (the tie count restarts)
    unsigned long long *tie_counter;
    RunningBest *run;        // device
    RunningBest *run_host;   // device-visible pinned host memory
    float *best_x;           // [m] row of the best
    float *win_v;            // its value (pinned host)
    int32_t *win_br;         // [K] its best responses (pinned host)
};

// One sweep launch.  Either (V_out, br_out) [evaluation mode: per-candidate outputs] or
// (blk_v, blk_i) [sweep mode: one record per workgroup] is used.
struct SweepArgs {
    const float *X;          // [count][m] fp32
    long long count;
    long long index_base;    // global index of row 0
    float *V_out;            // [count]            (evaluation mode, nullable)
    int32_t *br_out;         // [count][K]         (evaluation mode, nullable)
    float *blk_v;            // [nblocks]          (sweep mode)
    long long *blk_i;        // [nblocks] global candidate index, LLONG_MAX if none
    unsigned long long *tie_counter;  // += number of (candidate,type) evaluations with a tie
    // Evaluation mode only: l_out [count][K] receives the leader payoffs l_t[j*_t] at the best
    // responses.  In the general matrix-core kernel this selects the type-sliced instantiation:
    // for a handful of rows the launch is split over the types as well (one workgroup walking
    // every type would leave the chip idle), and a second kernel forms V_out from l_out in type
    // order (the same sum, term by term, as the unsliced kernel).
    float *l_out;
    int slice_stages;        // LDS stages per slice (set by the launcher)
    // Small-game kernel only, gen != 0: X is not read; row c is the flat-Dirichlet row
    // gen_first + c of the generator keyed (gen_k0, gen_k1), produced in registers with the
    // arithmetic of the generation kernel (sweep mode only).
    int gen;
    unsigned gen_k0, gen_k1;
    long long gen_first;
    SmallSweep small;        // small-game kernel, sweep mode
};

// Running best of one prior of a prior batch.
struct PriorBest {
    float value;
    int   has;
    long long index;
};

enum PathKind { PATH_VALU = 1, PATH_MFMA_F32 = 2, PATH_MFMA_BF16 = 3, PATH_MFMA_SPLIT = 4 };

// --- launchers (each validates nothing: the API layer has checked shapes) ----------------
// Number of workgroup records the sweep-mode launch of `count` candidates writes.
long long valu_num_blocks(long long count);
hipError_t launch_sweep_valu(const GameView &g, const SweepArgs &a, bool eval, hipStream_t s);

// Matrix-core variants.  mode: 0 = fp32 MFMA on fp32 payoffs, 1 = bf16 MFMA on bf16-rounded
// operands, 2 = bf16 MFMA on fp32 operands split into bf16 parts.  `exact` = every payoff is
// exactly representable in bf16 (lets mode 2 use three terms instead of six).  Returns a
// variant id >= 0, or -1 when the shape has no such kernel.
int mfma_select(int m, int n, int K, int mode, bool exact);
const char *mfma_variant_name(int variant);
long long mfma_num_blocks(int variant, long long count);
hipError_t launch_sweep_mfma(const GameView &g, const SweepArgs &a, hipStream_t s);
hipError_t mfma_prepare(int variant, int K);   // per game, on its device, before the first launch
bool mfma_slices_types(int variant);   // the variant honours SweepArgs::l_out
bool mfma_is_small(int variant);       // the small-game kernel: launch_finish_small applies
// Host-side packing of payoffs for a variant; returns malloc'ed buffers (caller frees).
void mfma_pack(int variant, int m, int n, int K, const float *A, const float *B, void **Bpack,
               size_t *Bbytes, void **ATpack, size_t *ATbytes, int *m_pad, int *n_pad);

// Small-game matrix-core kernel (n = 8, m = 8, K in {4, 8, 12, 16}, fp32); part of the MFMA path.
bool small_supported(int m, int n, int K, int storage);
long long small_num_blocks(long long count);
hipError_t launch_sweep_small(const GameView &g, const SweepArgs &a, hipStream_t s);
int small_num_slots();
hipError_t launch_finish_small(const GameView &g, const FinishArgs &f, hipStream_t s);
void small_pack(int m, int n, int K, const float *A, const float *B, void **Bpack, size_t *Bbytes,
                void **ATpack, size_t *ATbytes);

// first != 0: the running best is replaced, not merged (start of a sweep).  tie_counter (the
// chunk's count, left by the sweep kernel) is folded into run->ties and cleared.  The merged
// record is also written to run_host (device-visible pinned host memory).
hipError_t launch_reduce_merge(const float *blk_v, const long long *blk_i, long long nblocks,
                               const float *X, long long index_base, int m, int first,
                               unsigned long long *tie_counter, RunningBest *run,
                               RunningBest *run_host, float *best_x, hipStream_t s);

// *p = 0 by a one-thread kernel (a fill node that is safe to capture in a graph).
hipError_t launch_clear_u64(unsigned long long *p, hipStream_t s);
// Zero `bytes` (a multiple of 16) at the 16-byte aligned device address p, by a kernel.
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s);

// Prior batch (see prior_batch.hip): V_p[c] = sum_t priors[p][t] * L[c][t] and the arg-max over c
// for each of P priors, merged into run[P] (first != 0: replaced).  blk_v / blk_i: workspace of
// prior_batch_blocks(count, P) * P records.
int prior_batch_blocks(long long count, int P);
hipError_t launch_prior_batch(const float *L, long long count, long long index_base, int K,
                              const float *priors_dev, int P, int first, float *blk_v,
                              long long *blk_i, PriorBest *run, hipStream_t s);
hipError_t launch_gather_rows(const float *X, const PriorBest *run, int P, int m, float *rows,
                              hipStream_t s);

// Top-k reduction (see topk.hip): one level turns `count` (value, index) elements (idx null: the
// index of element e is index_base + e) into k records per workgroup, best first; an index of
// LLONG_MAX marks an empty record.  topk_level_blocks(count) workgroups.
long long topk_level_blocks(long long count);
hipError_t launch_topk_level(const float *vals, const long long *idx, long long count,
                             long long index_base, int k, float *out_v, long long *out_i,
                             hipStream_t s);
hipError_t launch_gather_indexed_rows(const float *X, const long long *idx, int rows, int m,
                                      float *out, hipStream_t s);

// Host code: the linear program of one pure follower profile (see profile_lp.hip).  Returns 0 with
// x_out[m] (on the simplex) and *value_out, 1 when the profile is a best response nowhere, 2 when
// the simplex method hit its iteration limit.  May throw std::bad_alloc.
int solve_profile_lp(int m, int n, int K, const float *A, const float *B, const float *prior,
                     const int32_t *profile, double *x_out, double *value_out);

// centre (device [m], nullable) and radius: the generated set shrunk towards the centre, each
// component fl(fl(radius * t) + fl(fl(1 - radius) * centre[i])); centre == nullptr: the plain set.
hipError_t launch_lattice(const unsigned long long *table, int m, int N, long long count,
                          const float *centre, float radius, float *out, hipStream_t s);
hipError_t launch_dirichlet(uint64_t seed, long long first, long long count, int m,
                            const float *centre, float radius, float *out, hipStream_t s);

}  // namespace bsse
