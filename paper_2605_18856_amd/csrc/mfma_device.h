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

// One step of the "which register holds the maximum" pass, pinned to four instructions:
//   vcc  = (u != gmax)                      v_cmp_neq_f32
//   idx  = vcc ? idx : JC                   v_cndmask_b32   (JC is an inline constant, 0..64:
//                                           a literal would be a second constant-bus read)
//   hits += number of lanes with u == gmax  s_bcnt0_i32_b64 + s_add_i32 (scalar unit)
// Written as one asm block so that the 64-bit compare mask lives only in vcc; left to the
// scheduler, the masks of many steps were kept alive at once and spilled.
template <int JC>
__device__ __forceinline__ void match_step(float u, float gmax, int &idx, int &hits)
{
    static_assert(JC >= 0 && JC <= 64, "must be an inline constant");
    int tmp;
    asm("v_cmp_neq_f32 vcc, %3, %4\n\t"
        "v_cndmask_b32 %0, %5, %0, vcc\n\t"
        "s_bcnt0_i32_b64 %2, vcc\n\t"
        "s_add_i32 %1, %1, %2"
        : "+v"(idx), "+s"(hits), "=&s"(tmp)
        : "v"(u), "v"(gmax), "i"(JC)
        : "vcc", "scc");
}

}  // namespace bsse
