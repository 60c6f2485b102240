// Candidate generation on the device (step 1 of the sweep): simplex-lattice unranking and
// seeded flat-Dirichlet rows.  Both kernels are write-bound: one coalesced pass over the
// output, no reads beyond a small table.
#include "bsse_internal.h"
#include "gen_device.h"

namespace bsse {

// Local sets: with a centre c (device, m floats) the generated point t is replaced by
// fl(fl(radius * t) + fl(omr * c)), omr = fl(1 - radius): the set shrunk by `radius` towards c.
// Separately rounded products and sum (no contraction), so the definition is three fp32 operations.
__device__ __forceinline__ float around(float t, const float *centre, int i, float radius, float omr)
{
#pragma clang fp contract(off)
    if (!centre) return t;
    const float a = radius * t, b = omr * centre[i];
    return a + b;
}

// ---------------------------------------------------------------------------------------
// Lattice.  Points are the compositions k of N into m parts in ascending lexicographic
// order.  table[q*(N+1) + R] = W(R, q) = C(R+q-1, q-1), the number of compositions of R
// into q parts (q = 1..m, R = 0..N).  With `rem` left to distribute over this part and q
// later parts, the compositions whose current part is < v number
//     S(v) = sum_{v'<v} W(rem-v', q) = W(rem, q+1) - W(rem-v, q+1)
// (hockey-stick identity), which is increasing in v, so the part is the largest v with
// S(v) <= rank, found by bisection.
__global__ void __launch_bounds__(256)
lattice_kernel(const unsigned long long *__restrict__ table, int m, int N, long long count,
               const float *__restrict__ centre, float radius, float omr, float *__restrict__ out)
{
    const float fN = (float)N;
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long r = (long long)blockIdx.x * blockDim.x + threadIdx.x; r < count; r += stride) {
        unsigned long long rr = (unsigned long long)r;
        int rem = N;
        float *row = out + r * m;
        for (int i = 0; i < m - 1; ++i) {
            const int q = m - 1 - i;
            const unsigned long long *Wq1 = table + (size_t)(q + 1) * (N + 1);
            const unsigned long long top = Wq1[rem];
            int lo = 0, hi = rem;
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (top - Wq1[rem - mid] <= rr) lo = mid; else hi = mid - 1;
            }
            rr -= top - Wq1[rem - lo];
            rem -= lo;
            row[i] = around((float)lo / fN, centre, i, radius, omr);   // IEEE division (correctly rounded)
        }
        row[m - 1] = around((float)rem / fN, centre, m - 1, radius, omr);
    }
}

hipError_t launch_lattice(const unsigned long long *table, int m, int N, long long count,
                          const float *centre, float radius, float *out, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    long long blocks = (count + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(lattice_kernel, dim3((unsigned)blocks), dim3(256), 0, s, table, m, N, count,
                       centre, radius, 1.0f - radius, out);
    return hipGetLastError();
}

// One thread per (row, group of four components): one Philox call, one float4 store, so a
// wavefront writes 1 KiB contiguously.  Requires m % 4 == 0 and m/4 a power of two <= 64, so
// that a row's threads sit in one wavefront and the row sum is a butterfly over them.
__global__ void __launch_bounds__(256)
dirichlet_quad_kernel(unsigned k0, unsigned k1, long long first, long long count, int m,
                      int log2_nb, const float *__restrict__ centre, float radius, float omr,
                      float *__restrict__ out)
{
    const int nb = 1 << log2_nb;
    const long long quads = count << log2_nb;
    const long long stride = (long long)gridDim.x * blockDim.x;
    const long long q0 = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    // all lanes of a wavefront iterate together (quads and stride are multiples of nb and the
    // trip count is uniform per row group), so the shuffles below see every partner lane
    for (long long base = q0 - threadIdx.x % 64; base < quads; base += stride) {
        const long long q = base + threadIdx.x % 64;
        const bool live = q < quads;
        const long long row = first + (q >> log2_nb);
        const unsigned b = (unsigned)(q & (nb - 1));
        float g0, g1, g2, g3;
        dirichlet_quad_raw(row, b, k0, k1, g0, g1, g2, g3);
        float sum = dirichlet_quad_sum(g0, g1, g2, g3);
        for (int d = 1; d < nb; d <<= 1) sum += __shfl_xor(sum, d, 64);
        dirichlet_quad_scale(sum, m, g0, g1, g2, g3);
        float4 v = make_float4(g0, g1, g2, g3);
        if (centre) {
            v.x = around(v.x, centre, 4 * b, radius, omr);     v.y = around(v.y, centre, 4 * b + 1, radius, omr);
            v.z = around(v.z, centre, 4 * b + 2, radius, omr); v.w = around(v.w, centre, 4 * b + 3, radius, omr);
        }
        if (live) reinterpret_cast<float4 *>(out)[q] = v;
    }
}

// Any m, any alignment: one thread per row, two passes over the generator (sum, then normalise).
// TREE (m a multiple of four with m/4 a power of two <= 64, the shapes the quad kernel takes): the
// row sum is formed in the quad kernel's order -- each quad as (g0 + g1) + (g2 + g3), then the
// quads pairwise level by level -- so that a row's bits do not depend on which kernel wrote it
// (the quad kernel needs a 16-byte aligned output; this one does not).
template <bool TREE>
__global__ void __launch_bounds__(256)
dirichlet_row_kernel(unsigned k0, unsigned k1, long long first, long long count, int m,
                     const float *__restrict__ centre, float radius, float omr, float *__restrict__ out)
{
#pragma clang fp contract(off)
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long r = (long long)blockIdx.x * blockDim.x + threadIdx.x; r < count; r += stride) {
        const long long row = first + r;
        const unsigned c0 = (unsigned)(unsigned long long)row;
        const unsigned c1 = (unsigned)((unsigned long long)row >> 32);
        const int nb = (m + 3) / 4;
        float sum = 0.0f;
        if (TREE) {
            float qs[64];
            for (int b = 0; b < nb; ++b) {
                float g0, g1, g2, g3;
                dirichlet_quad_raw(row, (unsigned)b, k0, k1, g0, g1, g2, g3);
                qs[b] = dirichlet_quad_sum(g0, g1, g2, g3);
            }
            for (int d = 1; d < nb; d <<= 1)
                for (int b = 0; b < nb; b += 2 * d) qs[b] = qs[b] + qs[b + d];
            sum = qs[0];
        } else {
            for (int b = 0; b < nb; ++b) {
                const U4 w = philox4x32_10(U4{ c0, c1, (unsigned)b, 0u }, k0, k1);
                const unsigned ww[4] = { w.x, w.y, w.z, w.w };
                for (int e = 0; e < 4; ++e)
                    if (4 * b + e < m) sum += unit_exponential(ww[e]);
            }
        }
        const float inv = sum > 0.0f ? 1.0f / sum : 0.0f;                // correctly rounded
        for (int b = 0; b < nb; ++b) {
            const U4 w = philox4x32_10(U4{ c0, c1, (unsigned)b, 0u }, k0, k1);
            const unsigned ww[4] = { w.x, w.y, w.z, w.w };
            for (int e = 0; e < 4; ++e)
                if (4 * b + e < m)
                    out[r * m + 4 * b + e] = around(
                        sum > 0.0f ? unit_exponential(ww[e]) * inv : 1.0f / (float)m, centre, 4 * b + e,
                        radius, omr);
        }
    }
}

hipError_t launch_dirichlet(uint64_t seed, long long first, long long count, int m,
                            const float *centre, float radius, float *out, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    const unsigned k0 = (unsigned)(seed & 0xFFFFFFFFull), k1 = (unsigned)(seed >> 32);
    int nb = m / 4, log2_nb = 0;
    while ((1 << log2_nb) < nb) ++log2_nb;
    const bool quad_shape = (m % 4 == 0) && nb >= 1 && (1 << log2_nb) == nb && nb <= 64;
    if (quad_shape && (uintptr_t)out % 16 == 0) {
        const long long quads = count * nb;
        long long blocks = (quads + 255) / 256;
        if (blocks > 256 * 32) blocks = 256 * 32;
        hipLaunchKernelGGL(dirichlet_quad_kernel, dim3((unsigned)blocks), dim3(256), 0, s, k0, k1,
                           first, count, m, log2_nb, centre, radius, 1.0f - radius, out);
    } else {
        long long blocks = (count + 255) / 256;
        if (blocks > 256 * 32) blocks = 256 * 32;
        if (quad_shape)
            hipLaunchKernelGGL(dirichlet_row_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, k0, k1,
                               first, count, m, centre, radius, 1.0f - radius, out);
        else
            hipLaunchKernelGGL(dirichlet_row_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, k0, k1,
                               first, count, m, centre, radius, 1.0f - radius, out);
    }
    return hipGetLastError();
}

}  // namespace bsse
