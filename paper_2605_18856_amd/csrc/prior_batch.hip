// Prior-robustness batch: the sweep for P priors at once.
//
// A follower's best response does not depend on the prior, so the leader payoffs at the best
// responses, L[c][t] = l_t[j*_t(x_c)], are computed once by the sweep kernels (evaluation mode
// with the per-type output) and every prior p only needs
//     V_p[c] = sum_t P[p][t] * L[c][t]        (fp32 fused multiply-adds, t ascending)
// and an arg-max over c (greatest value, lowest index).  Here priors sit on the lanes: lane
// (p, s) carries prior p of the current group of up to 64 priors and candidate stream s, keeps a
// running best over its candidates, and the streams, wavefronts and workgroups are folded at the
// end, so the per-candidate cost is K multiply-adds per 64 priors.
#include "bsse_internal.h"
#include <limits.h>

namespace bsse {

namespace {

constexpr int PB_WAVES = 4;

__device__ __forceinline__ bool pb_better(float v, long long i, float bv, long long bi)
{
    return v > bv || (v == bv && i < bi);
}

// blk_v / blk_i: [gridDim.x][P] records.  pri_lds != 0: the group's priors are staged in LDS as
// [t][64]; otherwise they are read from global memory.
__global__ void __launch_bounds__(PB_WAVES * 64)
prior_batch_kernel(const float *__restrict__ L, long long count, long long index_base, int K,
                   const float *__restrict__ priors, int P, int log2_pp, int pri_lds,
                   float *__restrict__ blk_v, long long *__restrict__ blk_i)
{
    extern __shared__ float pri[];                       // [K][64] when pri_lds
    __shared__ float sv[PB_WAVES][64];
    __shared__ long long si[PB_WAVES][64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pp = 1 << log2_pp;                         // priors per wavefront (power of two <= 64)
    const int streams = 64 >> log2_pp;                   // candidate streams per wavefront
    const int pl = lane & (pp - 1), s = lane >> log2_pp;
    const long long wave_id = (long long)blockIdx.x * PB_WAVES + wave;
    const long long step = (long long)gridDim.x * PB_WAVES * streams;

    for (int p0 = 0; p0 < P; p0 += pp) {
        const int p = p0 + pl;
        const bool live = p < P;
        if (pri_lds) {
            __syncthreads();                             // the previous group's readers are done
            for (int e = tid; e < K * 64; e += PB_WAVES * 64) {
                const int t = e >> 6, q = e & 63;
                pri[e] = (q < pp && p0 + q < P) ? priors[(size_t)(p0 + q) * K + t] : 0.0f;
            }
            __syncthreads();
        }
        float bv = -INFINITY;
        long long bi = LLONG_MAX;
        const long long c_first = wave_id * streams + s;
        if (pri_lds && (K & 3) == 0) {
            // U candidates in flight per lane: their row loads are independent, so the memory
            // latency is paid once per batch, not once per candidate
            constexpr int U = 8;
            const int K4 = K >> 2;
            for (long long cb = c_first; cb < count; cb += step * U) {
                float v[U];
                const float4 *row[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const long long c = cb + u * step;
                    row[u] = reinterpret_cast<const float4 *>(L + (c < count ? c : cb) * K);
                    v[u] = 0.0f;
                }
                for (int t4 = 0; t4 < K4; ++t4) {
                    float4 l[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) l[u] = row[u][t4];
                    const float q0 = pri[(4 * t4) * 64 + pl], q1 = pri[(4 * t4 + 1) * 64 + pl];
                    const float q2 = pri[(4 * t4 + 2) * 64 + pl], q3 = pri[(4 * t4 + 3) * 64 + pl];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        v[u] = fmaf(q0, l[u].x, v[u]); v[u] = fmaf(q1, l[u].y, v[u]);
                        v[u] = fmaf(q2, l[u].z, v[u]); v[u] = fmaf(q3, l[u].w, v[u]);
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const long long c = cb + u * step;
                    float x = v[u];
                    if (!(x == x)) x = -INFINITY;
                    if (live && c < count && x > bv) { bv = x; bi = index_base + c; }   // ascending
                }
            }
        } else {
            for (long long c = c_first; c < count; c += step) {
                const float *row = L + c * K;
                float v = 0.0f;
                if (pri_lds) {
                    for (int t = 0; t < K; ++t) v = fmaf(pri[t * 64 + pl], row[t], v);
                } else if (live) {
                    const float *pr = priors + (size_t)p * K;
                    for (int t = 0; t < K; ++t) v = fmaf(pr[t], row[t], v);
                }
                if (!(v == v)) v = -INFINITY;
                if (live && v > bv) { bv = v; bi = index_base + c; }   // a lane's candidates ascend
            }
        }
        // fold the streams of the wavefront, then the wavefronts
        for (int d = pp; d < 64; d <<= 1) {
            const float ov = __shfl_xor(bv, d, 64);
            const long long oi = __shfl_xor(bi, d, 64);
            if (pb_better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
        }
        sv[wave][lane] = bv; si[wave][lane] = bi;
        __syncthreads();
        if (wave == 0 && lane < pp && live) {
            for (int w = 1; w < PB_WAVES; ++w)
                if (pb_better(sv[w][lane], si[w][lane], bv, bi)) { bv = sv[w][lane]; bi = si[w][lane]; }
            blk_v[(size_t)blockIdx.x * P + p] = bv;
            blk_i[(size_t)blockIdx.x * P + p] = bi;
        }
        __syncthreads();
    }
}

// One workgroup per prior folds the records of all workgroups and merges into the running best
// of that prior (greater value, then lower index).
__global__ void __launch_bounds__(256)
prior_fold_kernel(const float *__restrict__ blk_v, const long long *__restrict__ blk_i, int nblocks,
                  int P, int first, PriorBest *__restrict__ run)
{
    __shared__ float sv[4];
    __shared__ long long si[4];
    const int p = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float bv = -INFINITY;
    long long bi = LLONG_MAX;
    for (int b = tid; b < nblocks; b += 256) {
        const float v = blk_v[(size_t)b * P + p];
        const long long i = blk_i[(size_t)b * P + p];
        if (pb_better(v, i, bv, bi)) { bv = v; bi = i; }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const float ov = __shfl_xor(bv, d, 64);
        const long long oi = __shfl_xor(bi, d, 64);
        if (pb_better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w)
            if (pb_better(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; }
        PriorBest r = run[p];
        if (first) { r.value = 0.0f; r.has = 0; r.index = -1; }
        if (bi != LLONG_MAX && (!r.has || bv > r.value || (bv == r.value && bi < r.index))) {
            r.value = bv; r.index = bi; r.has = 1;
        }
        run[p] = r;
    }
}

// rows[p][0..m) = X[index of prior p's winner] (row 0 when a prior has none)
__global__ void gather_rows_kernel(const float *__restrict__ X, const PriorBest *__restrict__ run,
                                   int P, int m, float *__restrict__ rows)
{
    const int p = blockIdx.x;
    const long long c = run[p].has ? run[p].index : 0;
    for (int i = threadIdx.x; i < m; i += blockDim.x) rows[(size_t)p * m + i] = X[c * m + i];
}

}  // namespace

int prior_batch_blocks(long long count, int P)
{
    int pp = 1;
    while (pp < P && pp < 64) pp <<= 1;
    const long long per_wg = (long long)PB_WAVES * (64 / pp);
    long long need = (count + per_wg - 1) / per_wg;
    // a few passes per lane amortise the fold; never more than one resident set
    need = (need + 7) / 8;
    if (need < 1) need = 1;
    return (int)(need < 1024 ? need : 1024);
}

hipError_t launch_prior_batch(const float *L, long long count, long long index_base, int K,
                              const float *priors_dev, int P, int first, float *blk_v,
                              long long *blk_i, PriorBest *run, hipStream_t s)
{
    if (count <= 0 || P <= 0) return hipSuccess;
    int log2_pp = 0;
    while ((1 << log2_pp) < P && log2_pp < 6) ++log2_pp;
    const int blocks = prior_batch_blocks(count, P);
    const size_t lds = (size_t)K * 64 * sizeof(float);
    const int pri_lds = lds <= 96 * 1024 ? 1 : 0;
    if (pri_lds && lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)prior_batch_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(prior_batch_kernel, dim3(blocks), dim3(PB_WAVES * 64), pri_lds ? lds : 0, s, L,
                       count, index_base, K, priors_dev, P, log2_pp, pri_lds, blk_v, blk_i);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(prior_fold_kernel, dim3(P), dim3(256), 0, s, blk_v, blk_i, blocks, P, first, run);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const float *X, const PriorBest *run, int P, int m, float *rows,
                              hipStream_t s)
{
    if (P <= 0) return hipSuccess;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(P), dim3(64), 0, s, X, run, P, m, rows);
    return hipGetLastError();
}

}  // namespace bsse
