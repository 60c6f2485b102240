// Device helpers shared by the matrix-core sweep kernels (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>

namespace bsse {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Row of a 32x32 MFMA accumulator tile held in register r of a lane, without the lane-half
// term 4*(lane/32): lane l holds column l%32 and rows 8*(r/4) + 4*(l/32) + r%4.
__device__ __host__ constexpr int acc_row_base(int r) { return 8 * (r / 4) + (r % 4); }

// max(a, b, c) / max(a, b) as single instructions.  (fmaxf() makes the compiler canonicalise
// every operand first -- one extra VALU instruction per input.)  NaN inputs are outside the
// contract; v_max3_f32 returns a non-NaN operand when there is one.
__device__ __forceinline__ float vmax3(float a, float b, float c)
{
    float d;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}
__device__ __forceinline__ float vmax2(float a, float b)
{
    float d;
    asm("v_max_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}

typedef __attribute__((address_space(3))) float lds_float;
typedef __attribute__((address_space(3))) unsigned char lds_byte;

// Partner-lane helpers built on v_permlane32_swap: the two results hold, in every lane, the
// value of the lane with the same column in the lower half and in the upper half, so any
// commutative combination of them is the pair's result, identical in both lanes.
__device__ __forceinline__ float pair_max(float v)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return vmax2(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ int pair_min(int v)
{
    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
    return min((int)r[0], (int)r[1]);
}
// The partner lane's value, through the LDS crossbar (no LDS memory is touched): this keeps
// the exchange off the vector ALU, where a swap costs two copies, the swap and a select.
// partner_addr = 4 * (lane ^ 32).
__device__ __forceinline__ float pair_other(float v, int partner_addr)
{
    return __uint_as_float((unsigned)__builtin_amdgcn_ds_bpermute(partner_addr, (int)__float_as_uint(v)));
}
__device__ __forceinline__ float pair_sum(float v)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Compile-time loop: f(integral_constant<int, I>) for I = Begin, Begin+Step, ... (Step may be
// negative), so that loop indices can feed immediate operands.
template <int I, int End, int Step, class F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr ((Step > 0 && I < End) || (Step < 0 && I > End)) {
        f(std::integral_constant<int, I>{});
        static_for<I + Step, End, Step>(f);
    }
}

// Four steps of the "which register holds the maximum" pass:
//     sum += sum_k (u_k == gmax ? c_k : 0),   k = 0..3
// where c_k = (action of register k) + 2^16, so that after all registers sum & 0xFFFF is the
// maximising action and sum >> 16 the number of maximisers (the action is only meaningful
// when that number is one; callers send every other case through an exact routine).
// Ten vector instructions for four values, nothing on the scalar unit.  Written as one asm
// block for two reasons: the four compare masks live in three scalar pairs plus vcc only
// inside the block (left to the scheduler, masks of many steps were kept alive and spilled),
// and every select stands three instructions behind its compare, which satisfies the two wait
// states this part needs between a vector write of a scalar register and a vector read of it.
__device__ __forceinline__ void match4(float u0, float u1, float u2, float u3, float gmax,
                                       unsigned c0, unsigned c1, unsigned c2, unsigned c3,
                                       unsigned &sum)
{
    unsigned t0, t1, t2, t3;
    unsigned long long m0, m1, m2;
    asm("v_cmp_eq_f32 %[m0], %[u0], %[g]\n\t"
        "v_cmp_eq_f32 %[m1], %[u1], %[g]\n\t"
        "v_cmp_eq_f32 %[m2], %[u2], %[g]\n\t"
        "v_cmp_eq_f32 vcc, %[u3], %[g]\n\t"
        "v_cndmask_b32 %[t0], 0, %[c0], %[m0]\n\t"
        "v_cndmask_b32 %[t1], 0, %[c1], %[m1]\n\t"
        "v_cndmask_b32 %[t2], 0, %[c2], %[m2]\n\t"
        "v_cndmask_b32 %[t3], 0, %[c3], vcc\n\t"
        "v_add3_u32 %[s], %[s], %[t0], %[t1]\n\t"
        "v_add3_u32 %[s], %[s], %[t2], %[t3]"
        : [s] "+v"(sum), [t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2), [t3] "=&v"(t3),
          [m0] "=&s"(m0), [m1] "=&s"(m1), [m2] "=&s"(m2)
        : [u0] "v"(u0), [u1] "v"(u1), [u2] "v"(u2), [u3] "v"(u3), [g] "v"(gmax),
          [c0] "v"(c0), [c1] "v"(c1), [c2] "v"(c2), [c3] "v"(c3)
        : "vcc");
}

// Four fp32 values as three bf16 parts each, x = x1 + x2 + x3: every part is the nearest bf16 of
// what is left, and what is left is formed exactly (a bf16 dot product with -1 in one slot and 0
// in the other subtracts one packed value from an fp32 number; the difference has at most 16
// significant bits).  p12 = (x1[0..3], x2[0..3]) and p31 = (x3[0..3], x1[0..3]) as eight bf16 each,
// the k-slot order of the small-game kernel's matrix instructions.
__device__ __forceinline__ void split_parts(const f32x4 &x, unsigned (&p12)[4], unsigned (&p31)[4])
{
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    // (-1, 0) and (0, -1) as packed bf16, kept in scalar registers as plain bit patterns: written
    // as constants they may be encoded as an inline operand of the dot instruction, and what that
    // operand expands to for a bf16 instruction is not something to rely on
    unsigned bits_lo = 0x0000BF80u, bits_hi = 0xBF800000u;
    asm("" : "+s"(bits_lo), "+s"(bits_hi));
    const v2bf minus_lo = __builtin_bit_cast(v2bf, bits_lo), minus_hi = __builtin_bit_cast(v2bf, bits_hi);
    // (a plain conversion, not inline asm: the compiler has to see the instruction to keep the
    // wait states between it and the dot products around it)
    auto pack = [](float a, float b) __attribute__((always_inline)) {
        typedef float v2f __attribute__((ext_vector_type(2)));
        const v2f ab = { a, b };
        return __builtin_bit_cast(unsigned, __builtin_convertvector(ab, v2bf));
    };
    auto rest = [&](unsigned packed, float a, float b, float &ra, float &rb) __attribute__((always_inline)) {
        const v2bf pv = __builtin_bit_cast(v2bf, packed);
        ra = __builtin_amdgcn_fdot2_f32_bf16(pv, minus_lo, a, false);
        rb = __builtin_amdgcn_fdot2_f32_bf16(pv, minus_hi, b, false);
    };
    float r[4], q[4];
    p12[0] = pack(x[0], x[1]); p12[1] = pack(x[2], x[3]);
    rest(p12[0], x[0], x[1], r[0], r[1]); rest(p12[1], x[2], x[3], r[2], r[3]);
    p12[2] = pack(r[0], r[1]); p12[3] = pack(r[2], r[3]);
    rest(p12[2], r[0], r[1], q[0], q[1]); rest(p12[3], r[2], r[3], q[2], q[3]);
    p31[0] = pack(q[0], q[1]); p31[1] = pack(q[2], q[3]);
    p31[2] = p12[0]; p31[3] = p12[1];
}

// Eight values and their maximum g: idx = the lowest position that holds g, n_eq = how many
// (lane, position) pairs of the wavefront hold g (64 exactly when every lane has one maximiser).
// Every compare mask lives in a scalar register pair (a select fed by vcc issues several times
// slower on this part), the position is a chain of selects between inline constants from the
// highest position down, and the count is taken on the scalar unit.  Each select stands at least
// two instructions behind its compare.
__device__ __forceinline__ void argmax8(float u0, float u1, float u2, float u3, float u4, float u5,
                                        float u6, float u7, float g, unsigned &idx, unsigned &n_eq)
{
    unsigned long long m0, m1, m2, m3, m4, m5, m6, m7;
    unsigned i, c, t;
    asm("v_cmp_eq_f32 %[m6], %[u6], %[g]\n\t"
        "v_cmp_eq_f32 %[m5], %[u5], %[g]\n\t"
        "v_cmp_eq_f32 %[m4], %[u4], %[g]\n\t"
        "v_cmp_eq_f32 %[m3], %[u3], %[g]\n\t"
        "v_cmp_eq_f32 %[m2], %[u2], %[g]\n\t"
        "v_cmp_eq_f32 %[m1], %[u1], %[g]\n\t"
        "v_cmp_eq_f32 %[m0], %[u0], %[g]\n\t"
        "v_cmp_eq_f32 %[m7], %[u7], %[g]\n\t"
        "v_cndmask_b32 %[i], 7, 6, %[m6]\n\t"
        "v_cndmask_b32 %[i], %[i], 5, %[m5]\n\t"
        "v_cndmask_b32 %[i], %[i], 4, %[m4]\n\t"
        "v_cndmask_b32 %[i], %[i], 3, %[m3]\n\t"
        "v_cndmask_b32 %[i], %[i], 2, %[m2]\n\t"
        "v_cndmask_b32 %[i], %[i], 1, %[m1]\n\t"
        "v_cndmask_b32 %[i], %[i], 0, %[m0]\n\t"
        "s_bcnt1_i32_b64 %[c], %[m0]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m1]\n\t"
        "s_add_u32 %[c], %[c], %[t]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m2]\n\t"
        "s_add_u32 %[c], %[c], %[t]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m3]\n\t"
        "s_add_u32 %[c], %[c], %[t]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m4]\n\t"
        "s_add_u32 %[c], %[c], %[t]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m5]\n\t"
        "s_add_u32 %[c], %[c], %[t]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m6]\n\t"
        "s_add_u32 %[c], %[c], %[t]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m7]\n\t"
        "s_add_u32 %[c], %[c], %[t]"
        : [i] "=&v"(i), [c] "=&s"(c), [t] "=&s"(t), [m0] "=&s"(m0), [m1] "=&s"(m1), [m2] "=&s"(m2),
          [m3] "=&s"(m3), [m4] "=&s"(m4), [m5] "=&s"(m5), [m6] "=&s"(m6), [m7] "=&s"(m7)
        : [u0] "v"(u0), [u1] "v"(u1), [u2] "v"(u2), [u3] "v"(u3), [u4] "v"(u4), [u5] "v"(u5),
          [u6] "v"(u6), [u7] "v"(u7), [g] "v"(g)
        : "scc");
    idx = i; n_eq = c;
}

// Eight follower payoffs u with their maximum g, and the eight leader payoffs w beside them:
// l = w at the lowest position where u holds g; n_eq = how many (lane, position) pairs of the
// wavefront hold g (64 exactly when every lane has one maximiser); with WANT_IDX also that
// position.  Compare masks in scalar pairs, selects from the highest position down, the count on
// the scalar unit, every select at least two instructions behind its compare.
template <bool WANT_IDX>
__device__ __forceinline__ void argmax8_pick(const float (&u)[8], const float (&w)[8], float g, float &l,
                                             unsigned &idx, unsigned &n_eq)
{
    unsigned long long m0, m1, m2, m3, m4, m5, m6, m7;
    unsigned c, t;
    float lv;
    asm("v_cmp_eq_f32 %[m6], %[u6], %[g]\n\t"
        "v_cmp_eq_f32 %[m5], %[u5], %[g]\n\t"
        "v_cmp_eq_f32 %[m4], %[u4], %[g]\n\t"
        "v_cmp_eq_f32 %[m3], %[u3], %[g]\n\t"
        "v_cmp_eq_f32 %[m2], %[u2], %[g]\n\t"
        "v_cmp_eq_f32 %[m1], %[u1], %[g]\n\t"
        "v_cmp_eq_f32 %[m0], %[u0], %[g]\n\t"
        "v_cmp_eq_f32 %[m7], %[u7], %[g]\n\t"
        "v_cndmask_b32 %[l], %[w7], %[w6], %[m6]\n\t"
        "v_cndmask_b32 %[l], %[l], %[w5], %[m5]\n\t"
        "v_cndmask_b32 %[l], %[l], %[w4], %[m4]\n\t"
        "v_cndmask_b32 %[l], %[l], %[w3], %[m3]\n\t"
        "v_cndmask_b32 %[l], %[l], %[w2], %[m2]\n\t"
        "v_cndmask_b32 %[l], %[l], %[w1], %[m1]\n\t"
        "v_cndmask_b32 %[l], %[l], %[w0], %[m0]\n\t"
        "s_bcnt1_i32_b64 %[c], %[m0]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m1]\n\t"
        "s_add_u32 %[c], %[c], %[t]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m2]\n\t"
        "s_add_u32 %[c], %[c], %[t]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m3]\n\t"
        "s_add_u32 %[c], %[c], %[t]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m4]\n\t"
        "s_add_u32 %[c], %[c], %[t]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m5]\n\t"
        "s_add_u32 %[c], %[c], %[t]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m6]\n\t"
        "s_add_u32 %[c], %[c], %[t]\n\t"
        "s_bcnt1_i32_b64 %[t], %[m7]\n\t"
        "s_add_u32 %[c], %[c], %[t]"
        : [l] "=&v"(lv), [c] "=&s"(c), [t] "=&s"(t), [m0] "=&s"(m0), [m1] "=&s"(m1), [m2] "=&s"(m2),
          [m3] "=&s"(m3), [m4] "=&s"(m4), [m5] "=&s"(m5), [m6] "=&s"(m6), [m7] "=&s"(m7)
        : [u0] "v"(u[0]), [u1] "v"(u[1]), [u2] "v"(u[2]), [u3] "v"(u[3]), [u4] "v"(u[4]), [u5] "v"(u[5]),
          [u6] "v"(u[6]), [u7] "v"(u[7]), [w0] "v"(w[0]), [w1] "v"(w[1]), [w2] "v"(w[2]), [w3] "v"(w[3]),
          [w4] "v"(w[4]), [w5] "v"(w[5]), [w6] "v"(w[6]), [w7] "v"(w[7]), [g] "v"(g)
        : "scc");
    l = lv; n_eq = c;
    if constexpr (WANT_IDX) {
        // (evaluation mode only: the position itself, by the same rule)
        unsigned i = 7u;
#pragma unroll
        for (int j = 6; j >= 0; --j) i = u[j] == g ? (unsigned)j : i;
        idx = i;
    }
}

// (bv, bc) <- (v, c) in the lanes where v > bv; the mask in a scalar register pair.
__device__ __forceinline__ void keep_greater2(float v, unsigned c, float &bv, unsigned &bc)
{
    unsigned long long m;
    asm("v_cmp_gt_f32 %[m], %[v], %[bv]\n\t"
        "s_nop 1\n\t"
        "v_cndmask_b32 %[bv], %[bv], %[v], %[m]\n\t"
        "v_cndmask_b32 %[bc], %[bc], %[c], %[m]"
        : [bv] "+v"(bv), [bc] "+v"(bc), [m] "=&s"(m)
        : [v] "v"(v), [c] "v"(c));
}

// (bv, bc, bp) <- (v, c, p) in the lanes where v > bv; the mask in a scalar register pair.
__device__ __forceinline__ void keep_greater(float v, unsigned c, unsigned p, float &bv, unsigned &bc,
                                             unsigned &bp)
{
    unsigned long long m;
    asm("v_cmp_gt_f32 %[m], %[v], %[bv]\n\t"
        "s_nop 1\n\t"
        "v_cndmask_b32 %[bv], %[bv], %[v], %[m]\n\t"
        "v_cndmask_b32 %[bc], %[bc], %[c], %[m]\n\t"
        "v_cndmask_b32 %[bp], %[bp], %[p], %[m]"
        : [bv] "+v"(bv), [bc] "+v"(bc), [bp] "+v"(bp), [m] "=&s"(m)
        : [v] "v"(v), [c] "v"(c), [p] "v"(p));
}

// The same for eight values in one asm block, and the running maximum over sixteen values in
// one block: the compiler pads every boundary between two asm statements with a no-op, so
// fewer, larger blocks save issue slots in the epilogue.
__device__ __forceinline__ void match8(const float *u, float gmax, const unsigned *c, unsigned &sum)
{
    unsigned t0, t1, t2, t3;
    unsigned long long m0, m1, m2;
    asm("v_cmp_eq_f32 %[m0], %[u0], %[g]\n\t"
        "v_cmp_eq_f32 %[m1], %[u1], %[g]\n\t"
        "v_cmp_eq_f32 %[m2], %[u2], %[g]\n\t"
        "v_cmp_eq_f32 vcc, %[u3], %[g]\n\t"
        "v_cndmask_b32 %[t0], 0, %[c0], %[m0]\n\t"
        "v_cndmask_b32 %[t1], 0, %[c1], %[m1]\n\t"
        "v_cndmask_b32 %[t2], 0, %[c2], %[m2]\n\t"
        "v_cndmask_b32 %[t3], 0, %[c3], vcc\n\t"
        "v_add3_u32 %[s], %[s], %[t0], %[t1]\n\t"
        "v_cmp_eq_f32 %[m0], %[u4], %[g]\n\t"
        "v_cmp_eq_f32 %[m1], %[u5], %[g]\n\t"
        "v_cmp_eq_f32 %[m2], %[u6], %[g]\n\t"
        "v_cmp_eq_f32 vcc, %[u7], %[g]\n\t"
        "v_add3_u32 %[s], %[s], %[t2], %[t3]\n\t"
        "v_cndmask_b32 %[t0], 0, %[c4], %[m0]\n\t"
        "v_cndmask_b32 %[t1], 0, %[c5], %[m1]\n\t"
        "v_cndmask_b32 %[t2], 0, %[c6], %[m2]\n\t"
        "v_cndmask_b32 %[t3], 0, %[c7], vcc\n\t"
        "v_add3_u32 %[s], %[s], %[t0], %[t1]\n\t"
        "v_add3_u32 %[s], %[s], %[t2], %[t3]"
        : [s] "+v"(sum), [t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2), [t3] "=&v"(t3),
          [m0] "=&s"(m0), [m1] "=&s"(m1), [m2] "=&s"(m2)
        : [u0] "v"(u[0]), [u1] "v"(u[1]), [u2] "v"(u[2]), [u3] "v"(u[3]), [u4] "v"(u[4]),
          [u5] "v"(u[5]), [u6] "v"(u[6]), [u7] "v"(u[7]), [g] "v"(gmax), [c0] "v"(c[0]),
          [c1] "v"(c[1]), [c2] "v"(c[2]), [c3] "v"(c[3]), [c4] "v"(c[4]), [c5] "v"(c[5]),
          [c6] "v"(c[6]), [c7] "v"(c[7])
        : "vcc");
}
// Compare pass as a bitmap: sixteen values against the maximum, bits = (bits << 16) | e with
// bit 15 - r of e set iff u[r] == gmax.  One compare and one add-with-carry (bits + bits + carry)
// per value; the four compares of a group precede the four adds that read their masks, which
// also keeps the two wait states a vector read of a vector-written scalar register needs.
__device__ __forceinline__ void bitmap16(const float *u, float gmax, unsigned &bits)
{
    unsigned long long m0, m1, m2;
#define BSSE_BM4(a, b, c, d)                                                    \
        "v_cmp_eq_f32 %[m0], %[u" #a "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m1], %[u" #b "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m2], %[u" #c "], %[g]\n\t"                              \
        "v_cmp_eq_f32 vcc, %[u" #d "], %[g]\n\t"                                \
        "v_addc_co_u32_e64 %[b], %[m0], %[b], %[b], %[m0]\n\t"                  \
        "v_addc_co_u32_e64 %[b], %[m1], %[b], %[b], %[m1]\n\t"                  \
        "v_addc_co_u32_e64 %[b], %[m2], %[b], %[b], %[m2]\n\t"                  \
        "v_addc_co_u32_e32 %[b], vcc, %[b], %[b], vcc\n\t"
    asm(BSSE_BM4(0, 1, 2, 3) BSSE_BM4(4, 5, 6, 7) BSSE_BM4(8, 9, 10, 11) BSSE_BM4(12, 13, 14, 15)
        : [b] "+v"(bits), [m0] "=&s"(m0), [m1] "=&s"(m1), [m2] "=&s"(m2)
        : [u0] "v"(u[0]), [u1] "v"(u[1]), [u2] "v"(u[2]), [u3] "v"(u[3]), [u4] "v"(u[4]),
          [u5] "v"(u[5]), [u6] "v"(u[6]), [u7] "v"(u[7]), [u8] "v"(u[8]), [u9] "v"(u[9]),
          [u10] "v"(u[10]), [u11] "v"(u[11]), [u12] "v"(u[12]), [u13] "v"(u[13]), [u14] "v"(u[14]),
          [u15] "v"(u[15]), [g] "v"(gmax)
        : "vcc");
#undef BSSE_BM4
}
// Two independent streams interleaved instruction by instruction: a wavefront that is alone in
// its epilogue (its neighbour on the SIMD being busy with MFMAs) issues dependent vector
// instructions at about half rate, independent ones at nearly full rate.
__device__ __forceinline__ void bitmap16x2(const float *ua, float ga, unsigned &ba, const float *ub,
                                           float gb, unsigned &bb)
{
    unsigned long long m0, m1, m2, m3, m4, m5, m6;
#define BSSE_BM4X2(a, b, c, d)                                                  \
        "v_cmp_eq_f32 %[m0], %[ua" #a "], %[ga]\n\t"                            \
        "v_cmp_eq_f32 %[m1], %[ub" #a "], %[gb]\n\t"                            \
        "v_cmp_eq_f32 %[m2], %[ua" #b "], %[ga]\n\t"                            \
        "v_cmp_eq_f32 %[m3], %[ub" #b "], %[gb]\n\t"                            \
        "v_cmp_eq_f32 %[m4], %[ua" #c "], %[ga]\n\t"                            \
        "v_cmp_eq_f32 %[m5], %[ub" #c "], %[gb]\n\t"                            \
        "v_cmp_eq_f32 %[m6], %[ua" #d "], %[ga]\n\t"                            \
        "v_cmp_eq_f32 vcc, %[ub" #d "], %[gb]\n\t"                              \
        "v_addc_co_u32_e64 %[ba], %[m0], %[ba], %[ba], %[m0]\n\t"               \
        "v_addc_co_u32_e64 %[bb], %[m1], %[bb], %[bb], %[m1]\n\t"               \
        "v_addc_co_u32_e64 %[ba], %[m2], %[ba], %[ba], %[m2]\n\t"               \
        "v_addc_co_u32_e64 %[bb], %[m3], %[bb], %[bb], %[m3]\n\t"               \
        "v_addc_co_u32_e64 %[ba], %[m4], %[ba], %[ba], %[m4]\n\t"               \
        "v_addc_co_u32_e64 %[bb], %[m5], %[bb], %[bb], %[m5]\n\t"               \
        "v_addc_co_u32_e64 %[ba], %[m6], %[ba], %[ba], %[m6]\n\t"               \
        "v_addc_co_u32_e32 %[bb], vcc, %[bb], %[bb], vcc\n\t"
#define BSSE_U4(x, a, b, c, d) [x##a] "v"(x[a]), [x##b] "v"(x[b]), [x##c] "v"(x[c]), [x##d] "v"(x[d])
    asm(BSSE_BM4X2(0, 1, 2, 3) BSSE_BM4X2(4, 5, 6, 7) BSSE_BM4X2(8, 9, 10, 11) BSSE_BM4X2(12, 13, 14, 15)
        : [ba] "+v"(ba), [bb] "+v"(bb), [m0] "=&s"(m0), [m1] "=&s"(m1), [m2] "=&s"(m2), [m3] "=&s"(m3),
          [m4] "=&s"(m4), [m5] "=&s"(m5), [m6] "=&s"(m6)
        : BSSE_U4(ua, 0, 1, 2, 3), BSSE_U4(ua, 4, 5, 6, 7), BSSE_U4(ua, 8, 9, 10, 11),
          BSSE_U4(ua, 12, 13, 14, 15), BSSE_U4(ub, 0, 1, 2, 3), BSSE_U4(ub, 4, 5, 6, 7),
          BSSE_U4(ub, 8, 9, 10, 11), BSSE_U4(ub, 12, 13, 14, 15), [ga] "v"(ga), [gb] "v"(gb)
        : "vcc");
#undef BSSE_BM4X2
}
// Sixteen values as two interleaved streams of eight (u[0..7] and u[8..15]) against one maximum:
// returns the 16-bit map with bit 15 - r set iff u[r] == gmax.
__device__ __forceinline__ unsigned bitmap16_split(const float *u, float gmax)
{
    unsigned ba = 0u, bb = 0u;
    unsigned long long m0, m1, m2, m3, m4, m5, m6;
#define BSSE_BM4S(a, b, c, d, e, f, g, h)                                       \
        "v_cmp_eq_f32 %[m0], %[u" #a "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m1], %[u" #e "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m2], %[u" #b "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m3], %[u" #f "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m4], %[u" #c "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m5], %[u" #g "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m6], %[u" #d "], %[g]\n\t"                              \
        "v_cmp_eq_f32 vcc, %[u" #h "], %[g]\n\t"                                \
        "v_addc_co_u32_e64 %[ba], %[m0], %[ba], %[ba], %[m0]\n\t"               \
        "v_addc_co_u32_e64 %[bb], %[m1], %[bb], %[bb], %[m1]\n\t"               \
        "v_addc_co_u32_e64 %[ba], %[m2], %[ba], %[ba], %[m2]\n\t"               \
        "v_addc_co_u32_e64 %[bb], %[m3], %[bb], %[bb], %[m3]\n\t"               \
        "v_addc_co_u32_e64 %[ba], %[m4], %[ba], %[ba], %[m4]\n\t"               \
        "v_addc_co_u32_e64 %[bb], %[m5], %[bb], %[bb], %[m5]\n\t"               \
        "v_addc_co_u32_e64 %[ba], %[m6], %[ba], %[ba], %[m6]\n\t"               \
        "v_addc_co_u32_e32 %[bb], vcc, %[bb], %[bb], vcc\n\t"
    asm(BSSE_BM4S(0, 1, 2, 3, 8, 9, 10, 11) BSSE_BM4S(4, 5, 6, 7, 12, 13, 14, 15)
        : [ba] "+v"(ba), [bb] "+v"(bb), [m0] "=&s"(m0), [m1] "=&s"(m1), [m2] "=&s"(m2), [m3] "=&s"(m3),
          [m4] "=&s"(m4), [m5] "=&s"(m5), [m6] "=&s"(m6)
        : [u0] "v"(u[0]), [u1] "v"(u[1]), [u2] "v"(u[2]), [u3] "v"(u[3]), [u4] "v"(u[4]),
          [u5] "v"(u[5]), [u6] "v"(u[6]), [u7] "v"(u[7]), [u8] "v"(u[8]), [u9] "v"(u[9]),
          [u10] "v"(u[10]), [u11] "v"(u[11]), [u12] "v"(u[12]), [u13] "v"(u[13]), [u14] "v"(u[14]),
          [u15] "v"(u[15]), [g] "v"(gmax)
        : "vcc");
#undef BSSE_BM4S
    return (ba << 8) | bb;
}
__device__ __forceinline__ void vmax_chain16x2(float &pa, const float *ua, float &pb, const float *ub)
{
#define BSSE_MX(a, b)                                                           \
        "v_max3_f32 %[pa], %[pa], %[ua" #a "], %[ua" #b "]\n\t"                  \
        "v_max3_f32 %[pb], %[pb], %[ub" #a "], %[ub" #b "]\n\t"
    asm(BSSE_MX(0, 1) BSSE_MX(2, 3) BSSE_MX(4, 5) BSSE_MX(6, 7) BSSE_MX(8, 9) BSSE_MX(10, 11)
        BSSE_MX(12, 13) BSSE_MX(14, 15)
        : [pa] "+v"(pa), [pb] "+v"(pb)
        : BSSE_U4(ua, 0, 1, 2, 3), BSSE_U4(ua, 4, 5, 6, 7), BSSE_U4(ua, 8, 9, 10, 11),
          BSSE_U4(ua, 12, 13, 14, 15), BSSE_U4(ub, 0, 1, 2, 3), BSSE_U4(ub, 4, 5, 6, 7),
          BSSE_U4(ub, 8, 9, 10, 11), BSSE_U4(ub, 12, 13, 14, 15));
#undef BSSE_MX
#undef BSSE_U4
}
// number of leading zero bits; 0xFFFFFFFF for zero
__device__ __forceinline__ unsigned ffbh(unsigned x)
{
    unsigned r;
    asm("v_ffbh_u32 %0, %1" : "=v"(r) : "v"(x));
    return r;
}
__device__ __forceinline__ float vmax_chain16(float p, const float *u)
{
    asm("v_max3_f32 %0, %0, %1, %2\n\t"
        "v_max3_f32 %0, %0, %3, %4\n\t"
        "v_max3_f32 %0, %0, %5, %6\n\t"
        "v_max3_f32 %0, %0, %7, %8\n\t"
        "v_max3_f32 %0, %0, %9, %10\n\t"
        "v_max3_f32 %0, %0, %11, %12\n\t"
        "v_max3_f32 %0, %0, %13, %14\n\t"
        "v_max3_f32 %0, %0, %15, %16"
        : "+v"(p)
        : "v"(u[0]), "v"(u[1]), "v"(u[2]), "v"(u[3]), "v"(u[4]), "v"(u[5]), "v"(u[6]), "v"(u[7]),
          "v"(u[8]), "v"(u[9]), "v"(u[10]), "v"(u[11]), "v"(u[12]), "v"(u[13]), "v"(u[14]), "v"(u[15]));
    return p;
}


// ---- helpers of the wide-game epilogue ---------------------------------------------------
// Maximum of sixteen values, two independent streams interleaved (no initial value needed: the
// first instruction of a stream takes three of its values).
__device__ __forceinline__ void vmax16x2_first(float &pa, const float *ua, float &pb, const float *ub)
{
#define BSSE_U4(x, a, b, c, d) [x##a] "v"(x[a]), [x##b] "v"(x[b]), [x##c] "v"(x[c]), [x##d] "v"(x[d])
#define BSSE_MX(a, b)                                                           \
        "v_max3_f32 %[pa], %[pa], %[ua" #a "], %[ua" #b "]\n\t"                  \
        "v_max3_f32 %[pb], %[pb], %[ub" #a "], %[ub" #b "]\n\t"
    asm("v_max3_f32 %[pa], %[ua0], %[ua1], %[ua2]\n\t"
        "v_max3_f32 %[pb], %[ub0], %[ub1], %[ub2]\n\t"
        BSSE_MX(3, 4) BSSE_MX(5, 6) BSSE_MX(7, 8) BSSE_MX(9, 10) BSSE_MX(11, 12) BSSE_MX(13, 14)
        "v_max_f32 %[pa], %[pa], %[ua15]\n\t"
        "v_max_f32 %[pb], %[pb], %[ub15]"
        : [pa] "=&v"(pa), [pb] "=&v"(pb)
        : BSSE_U4(ua, 0, 1, 2, 3), BSSE_U4(ua, 4, 5, 6, 7), BSSE_U4(ua, 8, 9, 10, 11),
          BSSE_U4(ua, 12, 13, 14, 15), BSSE_U4(ub, 0, 1, 2, 3), BSSE_U4(ub, 4, 5, 6, 7),
          BSSE_U4(ub, 8, 9, 10, 11), BSSE_U4(ub, 12, 13, 14, 15));
#undef BSSE_MX
#undef BSSE_U4
}
// Element-wise maximum over four vectors of sixteen: w[r] = max(a[r], b[r], c[r], d[r]).
__device__ __forceinline__ void vmax4x16(float *w, const float *a, const float *b, const float *c, const float *d)
{
#define BSSE_W4(x, i) [x##0] "v"(x[i]), [x##1] "v"(x[i + 1]), [x##2] "v"(x[i + 2]), [x##3] "v"(x[i + 3])
#pragma unroll
    for (int i = 0; i < 16; i += 4)
        asm("v_max3_f32 %[w0], %[a0], %[b0], %[c0]\n\t"
            "v_max3_f32 %[w1], %[a1], %[b1], %[c1]\n\t"
            "v_max3_f32 %[w2], %[a2], %[b2], %[c2]\n\t"
            "v_max3_f32 %[w3], %[a3], %[b3], %[c3]\n\t"
            "v_max_f32 %[w0], %[w0], %[d0]\n\t"
            "v_max_f32 %[w1], %[w1], %[d1]\n\t"
            "v_max_f32 %[w2], %[w2], %[d2]\n\t"
            "v_max_f32 %[w3], %[w3], %[d3]"
            : [w0] "=&v"(w[i]), [w1] "=&v"(w[i + 1]), [w2] "=&v"(w[i + 2]), [w3] "=&v"(w[i + 3])
            : BSSE_W4(a, i), BSSE_W4(b, i), BSSE_W4(c, i), BSSE_W4(d, i));
}
// w[r] = max(a[r], b[r])
__device__ __forceinline__ void vmax2x16(float *w, const float *a, const float *b)
{
#pragma unroll
    for (int i = 0; i < 16; i += 4)
        asm("v_max_f32 %[w0], %[a0], %[b0]\n\t"
            "v_max_f32 %[w1], %[a1], %[b1]\n\t"
            "v_max_f32 %[w2], %[a2], %[b2]\n\t"
            "v_max_f32 %[w3], %[a3], %[b3]"
            : [w0] "=&v"(w[i]), [w1] "=&v"(w[i + 1]), [w2] "=&v"(w[i + 2]), [w3] "=&v"(w[i + 3])
            : BSSE_W4(a, i), BSSE_W4(b, i));
#undef BSSE_W4
}
// bitmap16_split with every compare mask in a scalar register pair (a vector instruction that
// takes its mask or carry from vcc issues several times slower on this part than one that takes
// it from a scalar pair).
__device__ __forceinline__ unsigned bitmap16_pairs(const float *u, float gmax)
{
    unsigned ba = 0u, bb = 0u;
    unsigned long long m0, m1, m2, m3, m4, m5, m6, m7;
#define BSSE_BM4S(a, b, c, d, e, f, g, h)                                       \
        "v_cmp_eq_f32 %[m0], %[u" #a "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m1], %[u" #e "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m2], %[u" #b "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m3], %[u" #f "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m4], %[u" #c "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m5], %[u" #g "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m6], %[u" #d "], %[g]\n\t"                              \
        "v_cmp_eq_f32 %[m7], %[u" #h "], %[g]\n\t"                              \
        "v_addc_co_u32_e64 %[ba], %[m0], %[ba], %[ba], %[m0]\n\t"               \
        "v_addc_co_u32_e64 %[bb], %[m1], %[bb], %[bb], %[m1]\n\t"               \
        "v_addc_co_u32_e64 %[ba], %[m2], %[ba], %[ba], %[m2]\n\t"               \
        "v_addc_co_u32_e64 %[bb], %[m3], %[bb], %[bb], %[m3]\n\t"               \
        "v_addc_co_u32_e64 %[ba], %[m4], %[ba], %[ba], %[m4]\n\t"               \
        "v_addc_co_u32_e64 %[bb], %[m5], %[bb], %[bb], %[m5]\n\t"               \
        "v_addc_co_u32_e64 %[ba], %[m6], %[ba], %[ba], %[m6]\n\t"               \
        "v_addc_co_u32_e64 %[bb], %[m7], %[bb], %[bb], %[m7]\n\t"
    asm(BSSE_BM4S(0, 1, 2, 3, 8, 9, 10, 11) BSSE_BM4S(4, 5, 6, 7, 12, 13, 14, 15)
        : [ba] "+v"(ba), [bb] "+v"(bb), [m0] "=&s"(m0), [m1] "=&s"(m1), [m2] "=&s"(m2), [m3] "=&s"(m3),
          [m4] "=&s"(m4), [m5] "=&s"(m5), [m6] "=&s"(m6), [m7] "=&s"(m7)
        : [u0] "v"(u[0]), [u1] "v"(u[1]), [u2] "v"(u[2]), [u3] "v"(u[3]), [u4] "v"(u[4]),
          [u5] "v"(u[5]), [u6] "v"(u[6]), [u7] "v"(u[7]), [u8] "v"(u[8]), [u9] "v"(u[9]),
          [u10] "v"(u[10]), [u11] "v"(u[11]), [u12] "v"(u[12]), [u13] "v"(u[13]), [u14] "v"(u[14]),
          [u15] "v"(u[15]), [g] "v"(gmax));
#undef BSSE_BM4S
    return (ba << 8) | bb;
}

// (a + b) over the two lanes of a candidate, same value in both (integers)
__device__ __forceinline__ unsigned pair_add_u32(unsigned v)
{
    const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return r[0] + r[1];
}

}  // namespace bsse
