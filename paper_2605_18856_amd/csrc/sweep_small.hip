// Fused sweep for small games (n = 8 follower actions, m = 8 leader actions, K a multiple of
// 4 up to 16 types, fp32): steps 2-5 in one persistent kernel that is bound by reading the
// candidate rows (32 bytes each) once.
//
// Matrix-core layout.  One 32x32 tile holds four types x eight actions as its 32 rows and 32
// candidates as its columns.  The rows are ordered on the host so that the 16 rows a lane
// receives (accumulator rows 8q + 4h + rr in register 4q + rr, h = lane/32) are the eight
// actions of two whole types, 2h and 2h + 1 of the tile: register r holds action r % 8 of the
// lane's type r / 8.  Each lane therefore finishes (candidate, type) pairs on its own --
// maximum, lowest maximising action, leader payoff -- with no cross-lane traffic; the two lane
// halves of a candidate cover different types and their partial leader values are added once at
// the end.
//
// The contraction runs on the bf16 matrix pipe at fp32 accuracy.  The fp32 matrix instruction
// shares the vector unit's multipliers (the two never ran at the same time in the counters),
// so its 8 cycles per candidate were added to the epilogue's vector work.  Instead each fp32
// operand is written as the sum of three bf16 parts (x = x1 + x2 + x3, round to nearest each
// time, the remainders exact) and the six part products that matter -- x1 b1, x2 b1, x1 b2,
// x2 b2, x3 b1, x1 b3; the others are below 2^-25 of the product -- fill the 48 k-slots of
// three 32x32x16 instructions (3 cycles per candidate, beside the vector unit, not in it).
// Slot order: instruction i, lane half kh, element e: part P_i (e < 4) or Q_i (e >= 4) of
// leader action 4 kh + (e % 4), so that a lane splits only the four components it already
// holds for the leader payoff.  The follower parts are split on the host and stay in
// registers for the kernel's life; the leader matrix sits in LDS, one padded row per (type,
// action), in fp32.
#include "bsse_internal.h"
#include "mfma_device.h"
#include "gen_device.h"
#include <limits.h>
#include <stdlib.h>
#include <string.h>

namespace bsse {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int SM_M = 8, SM_N = 8;
constexpr int SM_WAVES = 4;
constexpr int SM_NT = 2;               // 32-candidate tiles per wavefront per iteration
constexpr int SM_AT_STRIDE = 12;       // floats per leader row in LDS (8 + pad: bank spread)
constexpr int SM_MAX_TILES = 4;

// TILES = K / 4 row tiles.  EVAL: per-candidate outputs instead of the workgroup record.
// Requires m == 8 and 16-byte aligned candidate rows (checked by the launcher).  The body of a
// workgroup; block / nblocks are its place in the (one-dimensional) grid of the pass.
template <int TILES, bool EVAL, bool GEN>
__device__ __forceinline__ void small_body(const GameView &g, const SweepArgs &a, unsigned block,
                                           unsigned nblocks)
{
    __shared__ __attribute__((aligned(16))) float at_lds[TILES * 4 * SM_N * SM_AT_STRIDE];
    __shared__ float red_v[SM_WAVES];
    __shared__ unsigned red_c[SM_WAVES];
    __shared__ unsigned red_p[SM_WAVES][2];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, col = lane & 31;
    const int K = g.K;
    const unsigned count = (unsigned)a.count;            // <= 2^31 per launch

    const unsigned per_iter = SM_NT * 32;
    const unsigned n_tasks = (count + per_iter - 1) / per_iter;
    const unsigned task0 = block * SM_WAVES + wave;
    const unsigned task_stride = nblocks * SM_WAVES;

    // candidate rows of one task: own = x[4h..4h+3] (the MFMA k-slots of this lane half),
    // oth = the other four components (needed for the leader payoff only).  Two sets of row
    // registers take turns: while one task is worked on, the rows of the wavefront's next task
    // land in the other set.  A task that lies wholly inside the range is addressed as a
    // wave-uniform base plus a fixed lane offset (no vector address arithmetic); the one ragged
    // task at the end of the range is done after the loop by the wavefront whose turn it is,
    // with the rows past the end reading the last row instead: they are evaluated like any
    // other and then left out of every result.
    const unsigned lane_own = (unsigned)(col * SM_M + 4 * h) * 4u;
    const unsigned lane_oth = (unsigned)(col * SM_M + 4 * (1 - h)) * 4u;
    auto load_task = [&](unsigned task, f32x4 (&own)[SM_NT], f32x4 (&oth)[SM_NT]) __attribute__((always_inline)) {
        const char *base = reinterpret_cast<const char *>(a.X) + (size_t)task * (per_iter * SM_M * 4);
#pragma unroll
        for (int ct = 0; ct < SM_NT; ++ct) {
            own[ct] = *(const f32x4 *)(base + ct * 32 * SM_M * 4 + lane_own);
            oth[ct] = *(const f32x4 *)(base + ct * 32 * SM_M * 4 + lane_oth);
        }
    };
    auto load_ragged = [&](unsigned task, f32x4 (&own)[SM_NT], f32x4 (&oth)[SM_NT]) __attribute__((always_inline)) {
#pragma unroll
        for (int ct = 0; ct < SM_NT; ++ct) {
            unsigned c = task * per_iter + ct * 32 + col;
            c = c < count ? c : count - 1u;
            const float *row = a.X + (size_t)c * SM_M;
            own[ct] = *(const f32x4 *)(row + 4 * h);
            oth[ct] = *(const f32x4 *)(row + 4 * (1 - h));
        }
    };
    const unsigned n_full = count / per_iter;            // tasks wholly inside the range
    // GEN: the rows are made here instead.  Lane half h produces components 4h..4h+3 of its
    // candidate (the thread (row, b = h) of the generation kernel); the row sum and the other four
    // components come from the partner lane.  Rows past the end of the range are ordinary rows of
    // the generator; they are left out of every result.
    const int partner_addr = 4 * (lane ^ 32);
    auto gen_task = [&](unsigned task, f32x4 (&own)[SM_NT], f32x4 (&oth)[SM_NT]) __attribute__((always_inline)) {
#pragma unroll
        for (int ct = 0; ct < SM_NT; ++ct) {
            const unsigned c = task * per_iter + ct * 32 + col;
            float g0, g1, g2, g3;
            dirichlet_quad_raw(a.gen_first + (long long)c, (unsigned)h, a.gen_k0, a.gen_k1, g0, g1, g2, g3);
            const float sum = pair_sum(dirichlet_quad_sum(g0, g1, g2, g3));
            dirichlet_quad_scale(sum, SM_M, g0, g1, g2, g3);
            own[ct] = f32x4{ g0, g1, g2, g3 };
#pragma unroll
            for (int k = 0; k < 4; ++k) oth[ct][k] = pair_other(own[ct][k], partner_addr);
        }
    };
    f32x4 own_a[SM_NT], oth_a[SM_NT], own_b[SM_NT], oth_b[SM_NT];
    if (!GEN && task0 < n_full) load_task(task0, own_a, oth_a);       // first rows in flight during set-up

    // leader rows -> LDS (packed on the host with the padded stride); follower fragments and
    // priors -> registers
    {
        const float *src = reinterpret_cast<const float *>(g.ATpack);
        for (int e = tid; e < TILES * 4 * SM_N * SM_AT_STRIDE; e += SM_WAVES * 64) at_lds[e] = src[e];
    }
    // per instruction: eight bf16 k-slots of this lane's tile row.  One row tile's fragments live
    // in registers for the kernel's life; with more tiles they are re-read from LDS at every
    // tile (registers for all of them cost spills in the loop).
    constexpr bool BF_LDS = TILES >= 2;
    __shared__ __attribute__((aligned(16))) u32x4 bf_lds[BF_LDS ? TILES * 3 * 64 : 1];
    u32x4 bfrag[BF_LDS ? 1 : TILES][3];
    float prior[TILES][2];
    const lds_float *rows_a[TILES][2];  // this lane's (type) leader rows, own-half columns
    int oth_delta;                      // float offset from own-half to other-half columns
    const lds_float *at_l = (const lds_float *)at_lds;
    {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(g.Bpack);
#pragma unroll
        for (int T = 0; T < TILES; ++T) {
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                if constexpr (BF_LDS) { if (wave == 0) bf_lds[(T * 3 + s) * 64 + lane] = src[(T * 3 + s) * 64 + lane]; }
                else bfrag[T][s] = src[(T * 3 + s) * 64 + lane];
            }
#pragma unroll
            for (int tl = 0; tl < 2; ++tl) {
                const int t = 4 * T + 2 * h + tl;
                prior[T][tl] = g.prior[t];
                rows_a[T][tl] = at_l + t * SM_N * SM_AT_STRIDE + 4 * h;
            }
        }
        oth_delta = 4 * (1 - h) - 4 * h;
    }
    // every set-up load has landed before the loop: the compiler would otherwise place its
    // waits for them at their first use, inside the loop, where they also wait for row requests
    __builtin_amdgcn_s_waitcnt(0x0F70);         // vmcnt(0)
    __syncthreads();

    float best_v = -INFINITY;
    unsigned best_c = 0xFFFFFFFFu;
    // best responses of the lane's best candidate, three bits each: this lane half's types only,
    // type 4T + 2h + tl at bits 3(2T + tl)
    unsigned best_pk = 0u;
    unsigned tie_count = 0;

    // One task: both candidate tiles and both of the lane's types advance together through one
    // straight-line block (four independent dependency chains for the scheduler to interleave);
    // the exact tie routine is a single rare branch per row tile.
    auto process = [&](unsigned task, bool full, const f32x4 (&xo)[SM_NT], const f32x4 (&xt)[SM_NT]) __attribute__((always_inline)) {
        const unsigned first = task * per_iter;
        float vhalf[SM_NT];
        unsigned pk[SM_NT];
        // the lane's four components as three bf16 parts: k-slots (x1, x2) for the instructions
        // against b1 and b2, (x3, x1) for the one against (b1, b3)
        u32x4 xs12[SM_NT], xs31[SM_NT];
#pragma unroll
        for (int ct = 0; ct < SM_NT; ++ct) {
            vhalf[ct] = 0.0f; pk[ct] = 0u;
            unsigned a12[4], a31[4];
            split_parts(xo[ct], a12, a31);
            xs12[ct] = u32x4{ a12[0], a12[1], a12[2], a12[3] };
            xs31[ct] = u32x4{ a31[0], a31[1], a31[2], a31[3] };
        }
#pragma unroll
        for (int T = 0; T < TILES; ++T) {
            f32x16 acc[SM_NT];
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[ct][r] = 0.0f;
            if constexpr (BF_LDS) {
#pragma unroll
                for (int s = 0; s < 3; ++s) bfrag[0][s] = bf_lds[(T * 3 + s) * 64 + lane];
            }
            const int TF = BF_LDS ? 0 : T;
            // smallest part products first
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct)
                acc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bfrag[TF][2]),
                                                                  __builtin_bit_cast(bf16x8, xs31[ct]), acc[ct], 0, 0, 0);
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct)
                acc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bfrag[TF][1]),
                                                                  __builtin_bit_cast(bf16x8, xs12[ct]), acc[ct], 0, 0, 0);
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct)
                acc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bfrag[TF][0]),
                                                                  __builtin_bit_cast(bf16x8, xs12[ct]), acc[ct], 0, 0, 0);

            // The asm blocks below read the accumulators, and the compiler's hazard handling does
            // not look into inline asm: no MFMA may sink below this point, and the wait states a
            // vector read of a fresh MFMA result needs (at most passes + 3 = 19) are explicit.
            // (the accumulators pass through the waiting block as operands, so that nothing that
            // reads them can be scheduled above it)
            __builtin_amdgcn_sched_barrier(0);
            static_assert(SM_NT == 2, "two accumulator tiles are named below");
            asm volatile("s_nop 15\n\ts_nop 3" : "+v"(acc[0]), "+v"(acc[1]));
            float gm[SM_NT][2], l[SM_NT][2];
            unsigned idx[SM_NT][2];
            unsigned n_eq = 0;          // wave-uniform: payoffs equal to their maximum, all four pairs
            auto leader = [&](int ct, int tl, unsigned j) __attribute__((always_inline)) {
                const lds_float *ra = rows_a[T][tl] + (int)j * SM_AT_STRIDE;
                const f32x4 qa = *(const __attribute__((address_space(3))) f32x4 *)ra;
                const f32x4 qb = *(const __attribute__((address_space(3))) f32x4 *)(ra + oth_delta);
                float v = xo[ct][0] * qa[0];
                v = fmaf(xo[ct][1], qa[1], v); v = fmaf(xo[ct][2], qa[2], v);
                v = fmaf(xo[ct][3], qa[3], v); v = fmaf(xt[ct][0], qb[0], v);
                v = fmaf(xt[ct][1], qb[1], v); v = fmaf(xt[ct][2], qb[2], v);
                v = fmaf(xt[ct][3], qb[3], v);
                return v;
            };
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct)
                static_for<0, 2, 1>([&](auto tlc) {
                    constexpr int tl = decltype(tlc)::value;
                    float m3 = vmax3(acc[ct][8 * tl], acc[ct][8 * tl + 1], acc[ct][8 * tl + 2]);
                    m3 = vmax3(m3, acc[ct][8 * tl + 3], acc[ct][8 * tl + 4]);
                    m3 = vmax3(m3, acc[ct][8 * tl + 5], acc[ct][8 * tl + 6]);
                    gm[ct][tl] = vmax2(m3, acc[ct][8 * tl + 7]);
                    unsigned eq;
                    argmax8(acc[ct][8 * tl], acc[ct][8 * tl + 1], acc[ct][8 * tl + 2], acc[ct][8 * tl + 3],
                            acc[ct][8 * tl + 4], acc[ct][8 * tl + 5], acc[ct][8 * tl + 6], acc[ct][8 * tl + 7],
                            gm[ct][tl], idx[ct][tl], eq);
                    n_eq += eq;
                });
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct)
#pragma unroll
                for (int tl = 0; tl < 2; ++tl) l[ct][tl] = leader(ct, tl, idx[ct][tl]);
            if (n_eq != 4u * SM_NT * 32u) {
                // Some lane has several maximisers (or none: a payoff that is not a number).
                // Exact, for the four pairs of every lane: maximisers in ascending action order,
                // leader payoff decides, then the lower action (lane-local; every lane owns its
                // (candidate, type) pairs).  A lane with one maximiser gets what it had.
#pragma unroll
                for (int ct = 0; ct < SM_NT; ++ct)
                    static_for<0, 2, 1>([&](auto tlc) {
                        constexpr int tl = decltype(tlc)::value;
                        const bool ok = first + ct * 32 + col < count;
                        float lbest = 0.0f;
                        unsigned jbest = 0;
                        int nm = 0;
#pragma unroll
                        for (int j = 0; j < SM_N; ++j)
                            if (acc[ct][8 * tl + j] == gm[ct][tl]) {
                                const float lj = leader(ct, tl, (unsigned)j);
                                if (nm == 0 || lj > lbest) { lbest = lj; jbest = (unsigned)j; }
                                ++nm;
                            }
                        l[ct][tl] = lbest; idx[ct][tl] = jbest;
                        tie_count += __builtin_popcountll(__builtin_amdgcn_ballot_w64(ok && nm >= 2));
                    });
            }
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct)
#pragma unroll
                for (int tl = 0; tl < 2; ++tl) {
                    vhalf[ct] = fmaf(prior[T][tl], l[ct][tl], vhalf[ct]);
                    if (!EVAL) pk[ct] |= idx[ct][tl] << (3 * (2 * T + tl));
                    if (EVAL) {
                        const unsigned c = first + ct * 32 + col;
                        if (a.br_out && c < count) a.br_out[(size_t)c * K + 4 * T + 2 * h + tl] = (int32_t)idx[ct][tl];
                        if (a.l_out && c < count) a.l_out[(size_t)c * K + 4 * T + 2 * h + tl] = l[ct][tl];
                    }
                }
        }
#pragma unroll
        for (int ct = 0; ct < SM_NT; ++ct) {
            const unsigned c = first + ct * 32 + col;
            float v = pair_sum(vhalf[ct]);
            if (EVAL) {
                if (!(v == v)) v = -INFINITY;
                if (a.V_out && c < count && h == 0) a.V_out[c] = v;
            } else {
                // a lane meets its candidates in ascending order: strictly greater replaces (a
                // value that is not a number compares false and is never recorded, and neither
                // is a row past the end of the range)
                if (!full) v = c < count ? v : -INFINITY;
                keep_greater(v, c, pk[ct], best_v, best_c, best_pk);
            }
        }
    };

    if (GEN) {
#pragma unroll 1
        for (unsigned task = task0; task < n_tasks; task += task_stride) {
            gen_task(task, own_a, oth_a);
            process(task, task < n_full, own_a, oth_a);
        }
    } else {
#pragma unroll 1
        for (unsigned task = task0; task < n_full; task += 2 * task_stride) {
            // (past the wavefront's last task the last whole task of the range is requested
            // once more: one shape of loop body, and the waits for rows never depend on the
            // position)
            const unsigned next = task + task_stride, last = n_full - 1u;
            load_task(next < last ? next : last, own_b, oth_b);
            process(task, true, own_a, oth_a);
            if (next >= n_full) break;
            load_task(next + task_stride < last ? next + task_stride : last, own_a, oth_a);
            process(next, true, own_b, oth_b);
        }
        if (n_full < n_tasks && n_full % task_stride == task0) {
            load_ragged(n_full, own_a, oth_a);
            process(n_full, false, own_a, oth_a);
        }
    }

    if (!EVAL) {
#pragma unroll
        for (int d = 16; d >= 1; d >>= 1) {          // both lane halves hold the same values
            const float ov = __shfl_xor(best_v, d, 64);
            const unsigned oc = __shfl_xor(best_c, d, 64);
            const unsigned op = __shfl_xor(best_pk, d, 64);
            if (ov > best_v || (ov == best_v && oc < best_c)) { best_v = ov; best_c = oc; best_pk = op; }
        }
        // lanes 0 and 32 now hold the same candidate, each with its half of the best responses
        if (lane == 0) { red_v[wave] = best_v; red_c[wave] = best_c; red_p[wave][0] = best_pk; }
        if (lane == 32) red_p[wave][1] = best_pk;
        __syncthreads();
        if (tid == 0) {
            int bw = 0;
            for (int w = 1; w < SM_WAVES; ++w)
                if (red_v[w] > best_v || (red_v[w] == best_v && red_c[w] < best_c)) {
                    best_v = red_v[w]; best_c = red_c[w]; bw = w;
                }
            // step 6: the workgroup's own running best over the chunks of this sweep (greater
            // value, then lower global index); nobody else touches the slot
            SmallSlot *slot = a.small.slots + block;
            const long long gi = a.index_base + (long long)best_c;
            if (best_c != 0xFFFFFFFFu &&
                (slot->epoch != a.small.epoch || best_v > slot->value ||
                 (best_v == slot->value && gi < slot->index))) {
                slot->value = best_v; slot->epoch = a.small.epoch; slot->index = gi;
                slot->br[0] = red_p[bw][0]; slot->br[1] = red_p[bw][1];
                if (GEN) {
                    float q[SM_M];
                    const long long row = a.gen_first + (long long)best_c;
                    dirichlet_quad_raw(row, 0u, a.gen_k0, a.gen_k1, q[0], q[1], q[2], q[3]);
                    dirichlet_quad_raw(row, 1u, a.gen_k0, a.gen_k1, q[4], q[5], q[6], q[7]);
                    const float sum = dirichlet_quad_sum(q[0], q[1], q[2], q[3]) + dirichlet_quad_sum(q[4], q[5], q[6], q[7]);
                    dirichlet_quad_scale(sum, SM_M, q[0], q[1], q[2], q[3]);
                    dirichlet_quad_scale(sum, SM_M, q[4], q[5], q[6], q[7]);
#pragma unroll
                    for (int i = 0; i < SM_M; ++i) slot->x[i] = q[i];
                } else {
                    const f32x4 *src = (const f32x4 *)(a.X + (size_t)best_c * SM_M);
                    *(f32x4 *)(slot->x) = src[0];
                    *(f32x4 *)(slot->x + 4) = src[1];
                }
            }
        }
        if (a.tie_counter && lane == 0 && tie_count) atomicAdd(a.tie_counter, (unsigned long long)tie_count);
    }
}

template <int TILES, bool EVAL>
__global__ void __launch_bounds__(SM_WAVES * 64, TILES == 1 ? 4 : 3)
sweep_small_kernel(GameView g, SweepArgs a)
{
    small_body<TILES, EVAL, false>(g, a, blockIdx.x, gridDim.x);
}

// The sweep over rows generated in registers (step 1 fused in): no candidate ever reaches memory.
template <int TILES>
__global__ void __launch_bounds__(SM_WAVES * 64, TILES == 1 ? 4 : 3)
sweep_small_gen_kernel(GameView g, SweepArgs a)
{
    small_body<TILES, false, true>(g, a, blockIdx.x, gridDim.x);
}

// Steps 5-6 at the end of a sweep: fold the slots of the current sweep (greatest value, lowest
// index among equals) and report the winner: value, index, tie count, row and best responses
// (unpacked from the slot; nothing is evaluated again).
__global__ void __launch_bounds__(SM_WAVES * 64)
small_finish_kernel(int K, FinishArgs f)
{
    __shared__ float sv[SM_WAVES];
    __shared__ long long si[SM_WAVES];
    __shared__ int sb[SM_WAVES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float bv = -INFINITY;
    long long bi = LLONG_MAX;
    int bb = -1;
    // (value, epoch and index are the first sixteen bytes of a slot: one load each, all of a
    // thread's loads independent of one another)
    for (int b = tid; b < f.nslots; b += SM_WAVES * 64) {
        const uint4 head = *reinterpret_cast<const uint4 *>(&f.slots[b]);
        const float v = __uint_as_float(head.x);
        const long long i = (long long)(((unsigned long long)head.w << 32) | head.z);
        if (head.y == f.epoch && (v > bv || (v == bv && i < bi))) { bv = v; bi = i; bb = b; }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const float ov = __shfl_xor(bv, d, 64);
        const long long oi = __shfl_xor(bi, d, 64);
        const int ob = __shfl_xor(bb, d, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; bb = ob; }
    }
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; sb[wave] = bb; }
    __syncthreads();
    if (tid != 0) return;
    for (int w = 1; w < SM_WAVES; ++w)
        if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) { bv = sv[w]; bi = si[w]; bb = sb[w]; }
    RunningBest r = *f.run;
    if (f.first) r.ties = 0ull;
    r.ties += *f.tie_counter;
    *f.tie_counter = 0ull;                       // counted; later chunks of the sweep add to zero
    r.has = bb >= 0 ? 1 : 0;
    r.value = bb >= 0 ? bv : 0.0f;
    r.index = bb >= 0 ? bi : -1;
    *f.run = r;
    *f.run_host = r;
    if (bb < 0) return;
    *f.win_v = bv;
    const unsigned p0 = f.slots[bb].br[0], p1 = f.slots[bb].br[1];
    for (int p = 0; 2 * p < K; ++p) {
        const int t = 4 * (p >> 1) + (p & 1);
        f.win_br[t] = (int32_t)((p0 >> (3 * p)) & 7u);          // lane half 0: types 4T, 4T+1
        f.win_br[t + 2] = (int32_t)((p1 >> (3 * p)) & 7u);      // lane half 1: types 4T+2, 4T+3
    }
    for (int i = 0; i < SM_M; ++i) f.best_x[i] = f.slots[bb].x[i];
}

typedef void (*small_kernel_t)(GameView, SweepArgs);
small_kernel_t small_kernel_for(int K, bool eval)
{
    switch (K / 4) {
    case 1: return eval ? sweep_small_kernel<1, true> : sweep_small_kernel<1, false>;
    case 2: return eval ? sweep_small_kernel<2, true> : sweep_small_kernel<2, false>;
    case 3: return eval ? sweep_small_kernel<3, true> : sweep_small_kernel<3, false>;
    case 4: return eval ? sweep_small_kernel<4, true> : sweep_small_kernel<4, false>;
    }
    return nullptr;
}

small_kernel_t small_gen_kernel_for(int K)
{
    switch (K / 4) {
    case 1: return sweep_small_gen_kernel<1>;
    case 2: return sweep_small_gen_kernel<2>;
    case 3: return sweep_small_gen_kernel<3>;
    case 4: return sweep_small_gen_kernel<4>;
    }
    return nullptr;
}

}  // namespace

bool small_supported(int m, int n, int K, int storage)
{
    return storage == 0 && n == SM_N && m == SM_M && K % 4 == 0 && K / 4 >= 1 && K / 4 <= SM_MAX_TILES;
}

// Persistent grid: one resident set of workgroups (per_cu per compute unit), never more than the work.
static long long small_blocks(long long count, int per_cu)
{
    const long long per_task = (long long)SM_NT * 32;
    const long long n_tasks = (count + per_task - 1) / per_task;
    const long long cap_waves = 256LL * per_cu * SM_WAVES;
    // every wavefront walks the same number of tasks (up to one): the grid is the smallest that
    // does the work in ceil(tasks / resident wavefronts) rounds, not the whole resident set
    const long long rounds = (n_tasks + cap_waves - 1) / cap_waves;
    const long long waves = rounds > 0 ? (n_tasks + rounds - 1) / rounds : 1;
    const long long blocks = (waves + SM_WAVES - 1) / SM_WAVES;
    return blocks < 1 ? 1 : blocks;
}
long long small_num_blocks(long long count) { return small_blocks(count, 4); }

hipError_t launch_sweep_small(const GameView &g, const SweepArgs &a, hipStream_t s)
{
    if (a.count <= 0) return hipSuccess;
    const bool eval = a.small.slots == nullptr;
    if (a.gen && eval) return hipErrorNotSupported;      // generated rows are swept, not listed
    small_kernel_t k = a.gen ? small_gen_kernel_for(g.K) : small_kernel_for(g.K, eval);
    if (!k) return hipErrorNotSupported;
    if (!a.gen && ((uintptr_t)a.X & 15) != 0) return hipErrorInvalidValue;   // the API layer checks alignment
    const int per_cu = 4;
    hipLaunchKernelGGL(k, dim3((unsigned)small_blocks(a.count, per_cu)), dim3(SM_WAVES * 64), 0, s, g, a);
    return hipGetLastError();
}

int small_num_slots() { return 256 * 5; }          // the largest grid launch_sweep_small uses

hipError_t launch_finish_small(const GameView &g, const FinishArgs &f, hipStream_t s)
{
    hipLaunchKernelGGL(small_finish_kernel, dim3(1), dim3(SM_WAVES * 64), 0, s, g.K, f);
    return hipGetLastError();
}

// fp32 -> nearest bf16 (ties to even), as the 16 high bits; and back.
static inline unsigned short bf16_rne_bits(float f)
{
    unsigned u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}
static inline float bf16_bits_to_float(unsigned short b)
{
    const unsigned u = (unsigned)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

// Host packing for the small-game kernel.
// Bpack: [tile][instruction i][lane][8] bf16; lane = 32*kh + r supplies, for tile row r = 8q +
// 4hh + rr (type t = 4*tile + 2*hh + q/2, action j = 4*(q%2) + rr), element e: the part of
// B_t[k = 4*kh + e%4][j] that instruction i multiplies in that slot: (b1, b1), (b2, b2), (b1, b3)
// for (e < 4, e >= 4) and i = 0, 1, 2, where b = b1 + b2 + b3 in bf16 parts.
// ATpack: [type][action][12] fp32: the leader column of (type, action) over the m leader
// actions, zero padded to 8, then 4 floats of padding.
void small_pack(int m, int n, int K, const float *A, const float *B, void **Bpack, size_t *Bbytes,
                void **ATpack, size_t *ATbytes)
{
    const int tiles = K / 4;
    *Bbytes = (size_t)tiles * 3 * 64 * 8 * sizeof(unsigned short);
    *ATbytes = (size_t)K * SM_N * SM_AT_STRIDE * sizeof(float);
    unsigned short *pb = (unsigned short *)calloc(*Bbytes, 1);
    float *pa = (float *)calloc(*ATbytes, 1);
    *Bpack = pb; *ATpack = pa;
    if (!pb || !pa) { free(pb); free(pa); *Bpack = nullptr; *ATpack = nullptr; return; }
    static const int part_of[3][2] = { { 0, 0 }, { 1, 1 }, { 0, 2 } };
    for (int T = 0; T < tiles; ++T)
        for (int lane = 0; lane < 64; ++lane) {
            const int kh = lane / 32, r = lane % 32;
            const int q = r / 8, hh = (r % 8) / 4, rr = r % 4;
            const int t = 4 * T + 2 * hh + q / 2, j = 4 * (q % 2) + rr;
            for (int e = 0; e < 8; ++e) {
                const int k = 4 * kh + e % 4;
                const float b = k < m ? B[((size_t)t * m + k) * n + j] : 0.0f;
                unsigned short part[3];
                part[0] = bf16_rne_bits(b);
                const float r1 = b - bf16_bits_to_float(part[0]);
                part[1] = bf16_rne_bits(r1);
                part[2] = bf16_rne_bits(r1 - bf16_bits_to_float(part[1]));
                for (int i = 0; i < 3; ++i)
                    pb[(((size_t)T * 3 + i) * 64 + lane) * 8 + e] = part[part_of[i][e / 4]];
            }
        }
    for (int t = 0; t < K; ++t)
        for (int j = 0; j < n; ++j)
            for (int i = 0; i < m; ++i)
                pa[((size_t)t * SM_N + j) * SM_AT_STRIDE + i] = A[((size_t)t * m + i) * n + j];
}

}  // namespace bsse
