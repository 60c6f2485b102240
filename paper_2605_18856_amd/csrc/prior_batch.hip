// Prior-robustness batch: the sweep for P priors at once.
//
// A follower's best response does not depend on the prior, so the leader payoffs at the best
// responses, L[c][t] = l_t[j*_t(x_c)], are computed once by the sweep kernels (evaluation mode
// with the per-type output) and every prior p only needs
//     V_p[c] = sum_t P[p][t] * L[c][t]        (fp32 fused multiply-adds, t ascending)
// and an arg-max over c (greatest value, lowest index).  Here priors sit on the lanes: lane
// (p, s) carries prior p of the current group of up to 64 priors and candidate stream s, keeps a
// running best over its candidates, and the streams, wavefronts and workgroups are folded at the
// end, so the per-candidate cost is K multiply-adds per 64 priors.  The rows of L reach the
// lanes through LDS (coalesced copy of a tile, then broadcast reads).
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
                   const float *__restrict__ priors, int P, int log2_pp, int pri_lds, int tile_rows,
                   float *__restrict__ blk_v, long long *__restrict__ blk_i)
{
    extern __shared__ __attribute__((aligned(16))) float pri[];   // [K][64] when pri_lds, then a tile of rows
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
        if (pri_lds && (K & 3) == 0) {
            // Rows go through LDS: the workgroup copies a tile of `tile_rows` rows with coalesced
            // 16-byte loads (every lane a different piece), and the wavefronts then read each row
            // as a broadcast from LDS, which costs the vector unit nothing.  (Loading the row a
            // wavefront works on straight from memory makes all 64 lanes fetch the same 16 bytes;
            // few such loads are in flight and the kernel sat waiting for memory.)
            float *rows = pri + K * 64;
            const int K4 = K >> 2;
            const long long ntiles = (count + tile_rows - 1) / tile_rows;
            int bo = -1;                                 // row of the lane's best so far (count <= 2^31)
            float q[16];                                 // the lane's prior, when K <= 16
#pragma unroll
            for (int t = 0; t < 16; ++t) q[t] = t < K ? pri[t * 64 + pl] : 0.0f;
            for (long long tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
                const long long r0 = tile * tile_rows;
                const int nr = (int)(count - r0 < tile_rows ? count - r0 : tile_rows);
                __syncthreads();                         // the previous tile's readers are done
                {
                    const float4 *src = reinterpret_cast<const float4 *>(L + r0 * K);
                    float4 *dst = reinterpret_cast<float4 *>(rows);
                    for (int e = tid; e < nr * K4; e += PB_WAVES * 64) dst[e] = src[e];
                }
                __syncthreads();
                // wavefront `wave`, stream s takes rows wave*streams + s, + PB_WAVES*streams, ...
                // (a NaN value never passes "v > best", so it needs no special case here)
                const int rstep = PB_WAVES * streams;
                int r = wave * streams + s;
                if (K4 <= 4) {
                    // the lane's prior in registers; four rows per trip
                    auto value = [&](int rr) __attribute__((always_inline)) {
                        const float4 *row = reinterpret_cast<const float4 *>(rows + (size_t)rr * K);
                        float v = 0.0f;
#pragma unroll
                        for (int t4 = 0; t4 < 4; ++t4) {
                            if (t4 >= K4) break;
                            const float4 l = row[t4];
                            v = fmaf(q[4 * t4], l.x, v); v = fmaf(q[4 * t4 + 1], l.y, v);
                            v = fmaf(q[4 * t4 + 2], l.z, v); v = fmaf(q[4 * t4 + 3], l.w, v);
                        }
                        return v;
                    };
                    for (; r + 3 * rstep < nr; r += 4 * rstep) {
                        const float v0 = value(r), v1 = value(r + rstep), v2 = value(r + 2 * rstep),
                                    v3 = value(r + 3 * rstep);
                        if (v0 > bv) { bv = v0; bo = (int)r0 + r; }
                        if (v1 > bv) { bv = v1; bo = (int)r0 + r + rstep; }
                        if (v2 > bv) { bv = v2; bo = (int)r0 + r + 2 * rstep; }
                        if (v3 > bv) { bv = v3; bo = (int)r0 + r + 3 * rstep; }
                    }
                    for (; r < nr; r += rstep) {
                        const float v = value(r);
                        if (v > bv) { bv = v; bo = (int)r0 + r; }
                    }
                } else {
                    for (; r < nr; r += rstep) {
                        const float4 *row = reinterpret_cast<const float4 *>(rows + (size_t)r * K);
                        float v = 0.0f;
                        for (int t4 = 0; t4 < K4; ++t4) {
                            const float4 l = row[t4];
                            v = fmaf(pri[(4 * t4) * 64 + pl], l.x, v);
                            v = fmaf(pri[(4 * t4 + 1) * 64 + pl], l.y, v);
                            v = fmaf(pri[(4 * t4 + 2) * 64 + pl], l.z, v);
                            v = fmaf(pri[(4 * t4 + 3) * 64 + pl], l.w, v);
                        }
                        if (v > bv) { bv = v; bo = (int)r0 + r; }
                    }
                }
            }
            if (live && bo >= 0) bi = index_base + bo;
            if (!live) bv = -INFINITY;
        } else {
            const long long c_first = wave_id * streams + s;
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
    const size_t lds_pri = (size_t)K * 64 * sizeof(float);
    const int pri_lds = lds_pri <= 96 * 1024 ? 1 : 0;
    // a tile of rows of about 8 KiB: small enough that the tiles outnumber the workgroups
    int tile_rows = 2048 / K;
    if (tile_rows < 4) tile_rows = 4;
    const size_t lds = pri_lds ? lds_pri + (size_t)tile_rows * K * sizeof(float) : 0;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)prior_batch_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(prior_batch_kernel, dim3(blocks), dim3(PB_WAVES * 64), lds, s, L,
                       count, index_base, K, priors_dev, P, log2_pp, pri_lds, tile_rows, blk_v, blk_i);
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
