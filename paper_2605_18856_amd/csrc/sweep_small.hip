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
// leader action 4 kh + (e % 4), so that a lane splits only the four components of its own lane
// half.  The leader payoffs of all eight actions of a (candidate, type) pair come off the matrix
// pipe the same way (three more instructions per tile, against the leader matrix in the same
// packing): the value at the best response is then a chain of selects under the masks of the
// arg-max compares, and nothing in the loop touches LDS or reads the other half of the row.
// Both matrices' parts are split on the host and stay in registers for the kernel's life.
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
constexpr int SM_MAX_TILES = 4;
#ifndef BSSE_SM_RING
#define BSSE_SM_RING 2
#endif
constexpr int SM_RING = BSSE_SM_RING;    // sets of row registers of the sweep over a buffer

// A 16-byte global load issued by hand (wave-uniform base, 32-bit lane offset, immediate offset)
// and the wait that makes the registers of two such loads usable: "at most PENDING vector memory
// operations outstanding", with the loaded values as operands so that nothing that uses them can
// be scheduled above the wait.  The compiler neither sees these loads nor waits for them: its own
// waits for rows in flight around a loop were "nothing outstanding" at the top of every trip.
template <int OFFSET> __device__ __forceinline__ void row_request(f32x4 &dst, unsigned lane_offset, const void *base)
{
    asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3" : "=v"(dst) : "v"(lane_offset), "s"(base), "n"(OFFSET));
}
template <int PENDING> __device__ __forceinline__ void rows_await(f32x4 &a, f32x4 &b)
{
    asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(PENDING));
}

// TILES = K / 4 row tiles.  EVAL: per-candidate outputs instead of the workgroup record.
// Requires m == 8 and 16-byte aligned candidate rows (checked by the launcher).  The body of a
// workgroup; block / nblocks are its place in the (one-dimensional) grid of the pass.
template <int TILES, bool EVAL, bool GEN>
__device__ __forceinline__ void small_body(const GameView &g, const SweepArgs &a, unsigned block,
                                           unsigned nblocks)
{
    __shared__ float red_v[SM_WAVES];
    __shared__ unsigned red_c[SM_WAVES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, col = lane & 31;
    const int K = g.K;
    const unsigned count = (unsigned)a.count;            // <= 2^31 per launch

    const unsigned per_iter = SM_NT * 32;
    const unsigned n_tasks = (count + per_iter - 1) / per_iter;
    const unsigned task0 = block * SM_WAVES + wave;
    const unsigned task_stride = nblocks * SM_WAVES;

    // candidate rows of one task: a lane holds x[4h..4h+3] of its candidate, the MFMA k-slots of
    // its lane half (the partner lane holds the other four; nothing else needs them).  Two sets of
    // row registers take turns: while one task is worked on, the rows of the wavefront's next
    // task land in the other set.  A task that lies wholly inside the range is addressed as a
    // wave-uniform base plus a fixed lane offset; the one ragged task at the end of the range is
    // done after the loop by the wavefront whose turn it is, with the rows past the end reading
    // the last row instead: they are evaluated like any other and then left out of every result.
    const unsigned lane_own = (unsigned)(col * SM_M + 4 * h) * 4u;
    auto load_task = [&](unsigned task, f32x4 (&own)[SM_NT]) __attribute__((always_inline)) {
        // (the task index is the same in every lane; said so, the base stays in scalar registers)
        const unsigned utask = (unsigned)__builtin_amdgcn_readfirstlane((int)task);
        const char *base = reinterpret_cast<const char *>(a.X) + (size_t)utask * (per_iter * SM_M * 4);
        static_assert(SM_NT == 2, "two tiles of rows are requested below");
        row_request<0>(own[0], lane_own, base);
        row_request<32 * SM_M * 4>(own[1], lane_own, base);
    };
    auto load_ragged = [&](unsigned task, f32x4 (&own)[SM_NT]) __attribute__((always_inline)) {
#pragma unroll
        for (int ct = 0; ct < SM_NT; ++ct) {
            unsigned c = task * per_iter + ct * 32 + col;
            c = c < count ? c : count - 1u;
            own[ct] = *(const f32x4 *)(a.X + (size_t)c * SM_M + 4 * h);
        }
    };
    const unsigned n_full = count / per_iter;            // tasks wholly inside the range
    // GEN: the rows are made here instead.  Lane half h produces components 4h..4h+3 of its
    // candidate (the thread (row, b = h) of the generation kernel); the row sum comes from the
    // pair.  Rows past the end of the range are ordinary rows of the generator; they are left out
    // of every result.
    auto gen_task = [&](unsigned task, f32x4 (&own)[SM_NT]) __attribute__((always_inline)) {
#pragma unroll
        for (int ct = 0; ct < SM_NT; ++ct) {
            const unsigned c = task * per_iter + ct * 32 + col;
            float g0, g1, g2, g3;
            dirichlet_quad_raw(a.gen_first + (long long)c, (unsigned)h, a.gen_k0, a.gen_k1, g0, g1, g2, g3);
            const float sum = pair_sum(dirichlet_quad_sum(g0, g1, g2, g3));
            dirichlet_quad_scale(sum, SM_M, g0, g1, g2, g3);
            own[ct] = f32x4{ g0, g1, g2, g3 };
        }
    };
    f32x4 ring[SM_RING][SM_NT];
    f32x4 (&own_a)[SM_NT] = ring[0];
    if (!GEN && task0 < n_full) load_task(task0, ring[0]);           // first rows in flight during set-up

    // per instruction: eight bf16 k-slots of this lane's tile row, follower payoffs (bfrag) and
    // leader payoffs (afrag) alike.  One row tile's fragments live in registers for the kernel's
    // life; with more tiles they are re-read from LDS at every tile (registers for all of them
    // cost spills in the loop).
    constexpr bool FR_LDS = TILES >= 2;
    __shared__ __attribute__((aligned(16))) u32x4 fr_lds[FR_LDS ? 2 * TILES * 3 * 64 : 1];
    u32x4 bfrag[FR_LDS ? 1 : TILES][3], afrag[FR_LDS ? 1 : TILES][3];
    float prior[TILES][2];
    {
        const u32x4 *srcb = reinterpret_cast<const u32x4 *>(g.Bpack);
        const u32x4 *srca = reinterpret_cast<const u32x4 *>(g.ATpack);
#pragma unroll
        for (int T = 0; T < TILES; ++T) {
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                if constexpr (FR_LDS) {
                    if (wave == 0) fr_lds[(T * 3 + s) * 64 + lane] = srcb[(T * 3 + s) * 64 + lane];
                    if (wave == 1) fr_lds[((TILES + T) * 3 + s) * 64 + lane] = srca[(T * 3 + s) * 64 + lane];
                } else {
                    bfrag[T][s] = srcb[(T * 3 + s) * 64 + lane];
                    afrag[T][s] = srca[(T * 3 + s) * 64 + lane];
                }
            }
#pragma unroll
            for (int tl = 0; tl < 2; ++tl) prior[T][tl] = g.prior[4 * T + 2 * h + tl];
        }
    }
    // every set-up load has landed before the loop: the compiler would otherwise place its
    // waits for them at their first use, inside the loop, where they also wait for row requests
    __builtin_amdgcn_s_waitcnt(0x0F70);         // vmcnt(0)
    __syncthreads();

    float best_v = -INFINITY;
    unsigned best_c = 0xFFFFFFFFu;
    unsigned tie_count = 0;

    // One task: both candidate tiles and both of the lane's types advance together through one
    // straight-line block (four independent dependency chains for the scheduler to interleave);
    // the exact tie routine is a single rare branch per row tile.
    auto process = [&](unsigned task, bool full, const f32x4 (&xo)[SM_NT]) __attribute__((always_inline)) {
        const unsigned first = task * per_iter;
        float vhalf[SM_NT];
        // the lane's four components as three bf16 parts: k-slots (x1, x2) for the instructions
        // against the first and second payoff parts, (x3, x1) for the one against (first, third)
        u32x4 xs12[SM_NT], xs31[SM_NT];
#pragma unroll
        for (int ct = 0; ct < SM_NT; ++ct) {
            vhalf[ct] = 0.0f;
            unsigned a12[4], a31[4];
            split_parts(xo[ct], a12, a31);
            xs12[ct] = u32x4{ a12[0], a12[1], a12[2], a12[3] };
            xs31[ct] = u32x4{ a31[0], a31[1], a31[2], a31[3] };
        }
#pragma unroll
        for (int T = 0; T < TILES; ++T) {
            if constexpr (FR_LDS) {
#pragma unroll
                for (int s = 0; s < 3; ++s) {
                    bfrag[0][s] = fr_lds[(T * 3 + s) * 64 + lane];
                    afrag[0][s] = fr_lds[((TILES + T) * 3 + s) * 64 + lane];
                }
            }
            const int TF = FR_LDS ? 0 : T;
            // follower payoffs u and leader payoffs w of the tile's 32 (type, action) rows, smallest
            // part products first
            f32x16 u[SM_NT], w[SM_NT];
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct)
#pragma unroll
                for (int r = 0; r < 16; ++r) { u[ct][r] = 0.0f; w[ct][r] = 0.0f; }
            auto mm = [](const u32x4 &fr, const u32x4 &xs, const f32x16 &c) __attribute__((always_inline)) {
                return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fr), __builtin_bit_cast(bf16x8, xs), c, 0, 0, 0);
            };
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct) u[ct] = mm(bfrag[TF][2], xs31[ct], u[ct]);
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct) u[ct] = mm(bfrag[TF][1], xs12[ct], u[ct]);
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct) u[ct] = mm(bfrag[TF][0], xs12[ct], u[ct]);
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct) w[ct] = mm(afrag[TF][2], xs31[ct], w[ct]);
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct) w[ct] = mm(afrag[TF][1], xs12[ct], w[ct]);
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct) w[ct] = mm(afrag[TF][0], xs12[ct], w[ct]);

            // The asm blocks below read the accumulators, and the compiler's hazard handling does
            // not look into inline asm: no MFMA may sink below this point, and the wait states a
            // vector read of a fresh MFMA result needs (at most passes + 3 = 19) are explicit.
            // (the accumulators pass through the waiting block as operands, so that nothing that
            // reads them can be scheduled above it)
            __builtin_amdgcn_sched_barrier(0);
            static_assert(SM_NT == 2, "two pairs of accumulator tiles are named below");
            asm volatile("s_nop 15\n\ts_nop 3" : "+v"(u[0]), "+v"(u[1]), "+v"(w[0]), "+v"(w[1]));
            float gm[SM_NT][2], l[SM_NT][2];
            unsigned idx[SM_NT][2];
            unsigned n_eq = 0;          // wave-uniform: payoffs equal to their maximum, all four pairs
#pragma unroll
            for (int ct = 0; ct < SM_NT; ++ct)
                static_for<0, 2, 1>([&](auto tlc) {
                    constexpr int tl = decltype(tlc)::value;
                    float m3 = vmax3(u[ct][8 * tl], u[ct][8 * tl + 1], u[ct][8 * tl + 2]);
                    m3 = vmax3(m3, u[ct][8 * tl + 3], u[ct][8 * tl + 4]);
                    m3 = vmax3(m3, u[ct][8 * tl + 5], u[ct][8 * tl + 6]);
                    gm[ct][tl] = vmax2(m3, u[ct][8 * tl + 7]);
                    unsigned eq;
                    float uu[8], ww[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) { uu[j] = u[ct][8 * tl + j]; ww[j] = w[ct][8 * tl + j]; }
                    idx[ct][tl] = 0u;
                    if (EVAL) argmax8_pick<true>(uu, ww, gm[ct][tl], l[ct][tl], idx[ct][tl], eq);
                    else argmax8_pick<false>(uu, ww, gm[ct][tl], l[ct][tl], idx[ct][tl], eq);
                    n_eq += eq;
                });
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
                            if (u[ct][8 * tl + j] == gm[ct][tl]) {
                                const float lj = w[ct][8 * tl + j];
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
                keep_greater2(v, c, best_v, best_c);
            }
        }
    };

    if (GEN) {
#pragma unroll 1
        for (unsigned task = task0; task < n_tasks; task += task_stride) {
            gen_task(task, own_a);
            process(task, task < n_full, own_a);
        }
    } else {
        // SM_RING sets of row registers: the rows of the wavefront's next SM_RING - 1 tasks are in
        // flight while one task is worked on (with one task in flight the loop was bound by the
        // latency of its loads, not by their bandwidth).  Past the wavefront's last task the last
        // whole task of the range is requested again: one shape of loop body, and the waits for
        // rows never depend on the position.
        const unsigned last = n_full > 0 ? n_full - 1u : 0u;
        auto request = [&](unsigned task, f32x4 (&own)[SM_NT]) __attribute__((always_inline)) {
            load_task(task < last ? task : last, own);
        };
        if (task0 < n_full) {
            static_for<1, SM_RING - 1, 1>([&](auto qc) {
                constexpr int q = decltype(qc)::value;
                request(task0 + q * task_stride, ring[q]);
            });
        }
#pragma unroll 1
        for (unsigned task = task0; task < n_full; task += SM_RING * task_stride) {
            bool done = false;
            static_for<0, SM_RING, 1>([&](auto qc) {
                constexpr int q = decltype(qc)::value;
                if (done) return;
                const unsigned mine = task + q * task_stride;
                if (mine >= n_full) { done = true; return; }
                request(mine + (SM_RING - 1) * task_stride, ring[(q + SM_RING - 1) % SM_RING]);
                // the SM_RING - 1 later tasks' loads (two each, issued in order) may stay in flight;
                // in evaluation mode stores are in flight as well, and everything is waited for
                rows_await<EVAL ? 0 : 2 * (SM_RING - 1)>(ring[q][0], ring[q][1]);
                process(mine, true, ring[q]);
            });
            if (done) break;
        }
        // nothing may still be on its way into registers that are about to mean something else
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (n_full < n_tasks && n_full % task_stride == task0) {
            load_ragged(n_full, own_a);
            process(n_full, false, own_a);
        }
    }

    if (!EVAL) {
#pragma unroll
        for (int d = 16; d >= 1; d >>= 1) {          // both lane halves hold the same values
            const float ov = __shfl_xor(best_v, d, 64);
            const unsigned oc = __shfl_xor(best_c, d, 64);
            if (ov > best_v || (ov == best_v && oc < best_c)) { best_v = ov; best_c = oc; }
        }
        if (lane == 0) { red_v[wave] = best_v; red_c[wave] = best_c; }
        __syncthreads();
        if (tid == 0) {
            for (int w2 = 1; w2 < SM_WAVES; ++w2)
                if (red_v[w2] > best_v || (red_v[w2] == best_v && red_c[w2] < best_c)) {
                    best_v = red_v[w2]; best_c = red_c[w2];
                }
            // step 6: the workgroup's own running best over the chunks of this sweep (greater
            // value, then lower global index); nobody else touches the slot.  The slot keeps the
            // row; the best responses of the sweep's winner are found at the end, by evaluating
            // that one row again.
            SmallSlot *slot = a.small.slots + block;
            const long long gi = a.index_base + (long long)best_c;
            if (best_c != 0xFFFFFFFFu &&
                (slot->epoch != a.small.epoch || best_v > slot->value ||
                 (best_v == slot->value && gi < slot->index))) {
                slot->value = best_v; slot->epoch = a.small.epoch; slot->index = gi;
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
// index among equals) and report the winner: value, index, tie count and row.  Its best
// responses come from a one-row evaluation launch behind this kernel (launch_finish_small): the
// same instruction sequence on the same row, hence the same decisions.
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
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // the winner's best responses: its row (left in best_x by the fold) through the evaluation
    // form of the sweep kernel; with no winner the row is whatever the buffer holds and the
    // responses are not reported
    SweepArgs ev{};
    ev.X = f.best_x; ev.count = 1; ev.br_out = f.win_br;
    small_kernel_t k = small_kernel_for(g.K, true);
    if (!k) return hipErrorNotSupported;
    hipLaunchKernelGGL(k, dim3(1), dim3(SM_WAVES * 64), 0, s, g, ev);
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
// Bpack and ATpack: [tile][instruction i][lane][8] bf16, follower and leader payoffs alike; lane =
// 32*kh + r supplies, for tile row r = 8q + 4hh + rr (type t = 4*tile + 2*hh + q/2, action
// j = 4*(q%2) + rr), element e: the part of P_t[k = 4*kh + e%4][j] that instruction i multiplies
// in that slot: (p1, p1), (p2, p2), (p1, p3) for (e < 4, e >= 4) and i = 0, 1, 2, where
// P = p1 + p2 + p3 in bf16 parts.
void small_pack(int m, int n, int K, const float *A, const float *B, void **Bpack, size_t *Bbytes,
                void **ATpack, size_t *ATbytes)
{
    const int tiles = K / 4;
    *Bbytes = (size_t)tiles * 3 * 64 * 8 * sizeof(unsigned short);
    *ATbytes = *Bbytes;
    unsigned short *pb = (unsigned short *)calloc(*Bbytes, 1);
    unsigned short *pa = (unsigned short *)calloc(*ATbytes, 1);
    *Bpack = pb; *ATpack = pa;
    if (!pb || !pa) { free(pb); free(pa); *Bpack = nullptr; *ATpack = nullptr; return; }
    static const int part_of[3][2] = { { 0, 0 }, { 1, 1 }, { 0, 2 } };
    for (int which = 0; which < 2; ++which) {
        const float *P = which ? A : B;
        unsigned short *out = which ? pa : pb;
        for (int T = 0; T < tiles; ++T)
            for (int lane = 0; lane < 64; ++lane) {
                const int kh = lane / 32, r = lane % 32;
                const int q = r / 8, hh = (r % 8) / 4, rr = r % 4;
                const int t = 4 * T + 2 * hh + q / 2, j = 4 * (q % 2) + rr;
                for (int e = 0; e < 8; ++e) {
                    const int k = 4 * kh + e % 4;
                    const float v = k < m ? P[((size_t)t * m + k) * n + j] : 0.0f;
                    unsigned short part[3];
                    part[0] = bf16_rne_bits(v);
                    const float r1 = v - bf16_bits_to_float(part[0]);
                    part[1] = bf16_rne_bits(r1);
                    part[2] = bf16_rne_bits(r1 - bf16_bits_to_float(part[1]));
                    for (int i = 0; i < 3; ++i)
                        out[(((size_t)T * 3 + i) * 64 + lane) * 8 + e] = part[part_of[i][e / 4]];
                }
            }
    }
}

}  // namespace bsse
