// Device code of the seeded flat-Dirichlet rows, shared by the generation kernels and by the
// sweep kernel that generates its candidates in registers (not installed).  Everything here is a
// fixed sequence of separately rounded fp32 operations (no contraction), so that every kernel that
// includes it produces the same bits for the same (seed, row).
#pragma once
#include <hip/hip_runtime.h>

namespace bsse {

// Philox4x32 with 10 rounds, from the description in Salmon, Moraes, Dror, Shaw (SC'11):
// two 32x32->64 multiplies per round feed a fixed permutation with key injection; the key
// advances by two Weyl constants between rounds.
struct U4 { unsigned x, y, z, w; };

__device__ __forceinline__ unsigned long long mul_wide(unsigned a, unsigned b)
{
    unsigned long long d;
    asm("v_mad_u64_u32 %0, vcc, %1, %2, 0" : "=v"(d) : "s"(a), "v"(b) : "vcc");
    return d;
}

__device__ __forceinline__ U4 philox4x32_10(U4 c, unsigned k0, unsigned k1)
{
#pragma unroll
    for (int rnd = 0; rnd < 10; ++rnd) {
        // one 32x32->64 multiply-add instruction per product (full rate on this part; the
        // compiler would otherwise issue separate high and low multiplies)
        const unsigned long long p0 = mul_wide(0xD2511F53u, c.x), p1 = mul_wide(0xCD9E8D57u, c.z);
        const unsigned hi0 = (unsigned)(p0 >> 32), lo0 = (unsigned)p0;
        const unsigned hi1 = (unsigned)(p1 >> 32), lo1 = (unsigned)p1;
        U4 d;
        d.x = hi1 ^ c.y ^ k0;
        d.y = lo1;
        d.z = hi0 ^ c.w ^ k1;
        d.w = lo0;
        c = d;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c;
}

// A 32-bit word to a unit exponential: u = ((w >> 8) + 1) / 2^24 is in (0, 1].
__device__ __forceinline__ float unit_exponential(unsigned w)
{
#pragma clang fp contract(off)
    const float u = (float)((w >> 8) + 1u) * 5.9604644775390625e-08f;   // exact: < 2^24+1
    // -ln u = -log2(u) * ln 2 with the product carried in two parts; u >= 2^-24 is never
    // subnormal, so the hardware logarithm needs no range scaling
    const float r = __builtin_amdgcn_logf(u);
    const float c = 0x1.62e42ep-1f, cc = 0x1.efa39ep-25f;                // ln 2 = c + cc
    const float y = r * c;
    return -(y + fmaf(r, cc, fmaf(r, c, -y)));
}

// The four unnormalised components 4b .. 4b+3 of row `row`: one generator call, counter
// (row low, row high, b, 0).
__device__ __forceinline__ void dirichlet_quad_raw(long long row, unsigned b, unsigned k0, unsigned k1,
                                                   float &g0, float &g1, float &g2, float &g3)
{
    const U4 c = { (unsigned)(unsigned long long)row, (unsigned)((unsigned long long)row >> 32), b, 0u };
    const U4 w = philox4x32_10(c, k0, k1);
    g0 = unit_exponential(w.x); g1 = unit_exponential(w.y);
    g2 = unit_exponential(w.z); g3 = unit_exponential(w.w);
}

// Sum of a quad in the order every kernel uses.
__device__ __forceinline__ float dirichlet_quad_sum(float g0, float g1, float g2, float g3)
{
#pragma clang fp contract(off)
    return (g0 + g1) + (g2 + g3);
}

// A quad of the normalised row from its unnormalised components and the row sum: g_i * fl(1/sum)
// (the division correctly rounded), or 1/m throughout when the sum is zero.
__device__ __forceinline__ void dirichlet_quad_scale(float sum, int m, float &g0, float &g1, float &g2,
                                                     float &g3)
{
#pragma clang fp contract(off)
    if (sum > 0.0f) {
        const float inv = 1.0f / sum;
        g0 = g0 * inv; g1 = g1 * inv; g2 = g2 * inv; g3 = g3 * inv;
    } else {
        g0 = g1 = g2 = g3 = 1.0f / (float)m;
    }
}

}  // namespace bsse
