// Fused sweep, plain-VALU path (steps 2-5 for any shape): one lane per candidate.
//
// Each 64-lane workgroup stages its 64 candidate rows in LDS with coalesced loads, then
// every lane walks types and follower actions.  Payoff addresses are uniform across the
// wavefront, so B and the prior arrive through scalar loads and every FMA has one SGPR
// operand; the only per-lane memory traffic is the LDS read of x[i] (stride chosen odd, so
// the 64 lanes hit distinct banks) and the rare leader-payoff column gathers.
// This path is the correct-for-every-shape baseline and the one used for small games; large
// games go through the MFMA path.
#include "bsse_internal.h"
#include <limits.h>

namespace bsse {

namespace {

constexpr int WG = 64;           // one wavefront per workgroup
constexpr int JB = 4;            // follower actions evaluated together
constexpr int MAX_STAGE_M = 255; // rows longer than this are read from global memory directly

__device__ __forceinline__ float round_bf16(float v)
{
    // nearest-even rounding of an fp32 value to bfloat16 precision (finite inputs)
    unsigned b = __float_as_uint(v);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return __uint_as_float(b & 0xFFFF0000u);
}

struct XRow {
    const float *p;     // LDS row or global row
    __device__ __forceinline__ float operator[](int i) const { return p[i]; }
};

// leader payoff of follower action j for type t: sum_i x[i]*A_t[i][j], i ascending
__device__ __forceinline__ float leader_dot(const GameView &g, const XRow &x, int t, int j)
{
    const float *col = g.AT + ((size_t)t * g.n + j) * g.m;
    float l = 0.0f;
    for (int i = 0; i < g.m; ++i) l = fmaf(x[i], col[i], l);
    return l;
}

template <bool EVAL>
__global__ void __launch_bounds__(WG) sweep_valu_kernel(GameView g, SweepArgs a)
{
    extern __shared__ float xs[];
    const int lane = threadIdx.x;
    const int m = g.m, n = g.n, K = g.K;
    const long long c0 = (long long)blockIdx.x * WG;
    const long long c = c0 + lane;
    const bool valid = c < a.count;
    const bool staged = m <= MAX_STAGE_M;
    const int ld = m | 1;                         // odd row stride: conflict-free per-lane rows

    XRow x;
    if (staged) {
        const long long rows = (a.count - c0 < WG) ? (a.count - c0) : WG;
        const long long total = rows * m;
        const float *src = a.X + c0 * m;
        for (long long e = lane; e < (long long)WG * m; e += WG) {
            float v = e < total ? src[e] : 0.0f;
            if (g.x_bf16) v = round_bf16(v);
            const int r = (int)(e / m), i = (int)(e % m);
            xs[r * ld + i] = v;
        }
        __syncthreads();
        x.p = xs + lane * ld;
    } else {
        // long rows: read straight from global memory (bf16 rounding is applied on use below)
        x.p = a.X + (valid ? c : 0) * m;
    }
    const bool round_on_use = !staged && g.x_bf16;

    float V = 0.0f;
    unsigned ties = 0;
    for (int t = 0; t < K; ++t) {
        const float *Bt = g.B + (size_t)t * m * n;
        float best_u = -INFINITY, best_l = 0.0f;
        int best_j = 0;
        bool has_l = false, tied = false;
        for (int j0 = 0; j0 < n; j0 += JB) {
            float u[JB];
#pragma unroll
            for (int q = 0; q < JB; ++q) u[q] = 0.0f;
            for (int i = 0; i < m; ++i) {
                float xi = x[i];
                if (round_on_use) xi = round_bf16(xi);
                const float *brow = Bt + (size_t)i * n + j0;
#pragma unroll
                for (int q = 0; q < JB; ++q)
                    if (j0 + q < n) u[q] = fmaf(xi, brow[q], u[q]);
            }
#pragma unroll
            for (int q = 0; q < JB; ++q) {
                const int j = j0 + q;
                if (j >= n) break;
                if (u[q] > best_u) {
                    best_u = u[q]; best_j = j; has_l = false; tied = false;
                } else if (u[q] == best_u) {
                    // exact follower tie: the leader's payoff decides, then the lower index
                    tied = true;
                    if (!has_l) { best_l = leader_dot(g, x, t, best_j); has_l = true; }
                    const float lj = leader_dot(g, x, t, j);
                    if (lj > best_l) { best_l = lj; best_j = j; }
                }
            }
        }
        if (!has_l) best_l = leader_dot(g, x, t, best_j);
        if (best_u == -INFINITY) tied = false;     // non-finite input: unspecified, not counted
        V = fmaf(g.prior[t], best_l, V);
        ties += tied ? 1u : 0u;
        if (EVAL && valid && a.br_out) a.br_out[c * K + t] = best_j;
        if (EVAL && valid && a.l_out) a.l_out[c * K + t] = best_l;
    }
    if (!(V == V)) V = -INFINITY;                  // NaN never wins

    if (EVAL) {
        if (valid && a.V_out) a.V_out[c] = V;
    } else {
        float bv = valid ? V : -INFINITY;
        long long bi = valid ? a.index_base + c : LLONG_MAX;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const float ov = __shfl_xor(bv, d, 64);
            const long long oi = __shfl_xor(bi, d, 64);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        if (lane == 0) { a.blk_v[blockIdx.x] = bv; a.blk_i[blockIdx.x] = bi; }
    }
    if (!valid) ties = 0;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) ties += __shfl_xor(ties, d, 64);
    if (lane == 0 && ties && a.tie_counter) atomicAdd(a.tie_counter, (unsigned long long)ties);
}

}  // namespace

long long valu_num_blocks(long long count) { return (count + WG - 1) / WG; }

hipError_t launch_sweep_valu(const GameView &g, const SweepArgs &a, bool eval, hipStream_t s)
{
    if (a.count <= 0) return hipSuccess;
    const long long blocks = valu_num_blocks(a.count);
    const size_t lds = g.m <= MAX_STAGE_M ? (size_t)WG * (g.m | 1) * sizeof(float) : 0;
    if (eval)
        hipLaunchKernelGGL(sweep_valu_kernel<true>, dim3((unsigned)blocks), dim3(WG), lds, s, g, a);
    else
        hipLaunchKernelGGL(sweep_valu_kernel<false>, dim3((unsigned)blocks), dim3(WG), lds, s, g, a);
    return hipGetLastError();
}

}  // namespace bsse
