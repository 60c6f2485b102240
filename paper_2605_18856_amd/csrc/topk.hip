// Top-k reduction over candidates: the k best (value, index) pairs in the order "greater value
// first, lower index among equal values" -- the order whose first element is the sweep's winner.
//
// One kernel, applied level by level.  A workgroup takes a slice of TK_SLICE elements into
// registers (TK_E per thread) and extracts its k best in k rounds: every thread keeps the best of
// its elements not yet taken, a shuffle/LDS reduction finds the workgroup's best (one barrier per
// round: the wavefronts' winners are double-buffered and every thread folds them itself), and only
// the owning thread rescans its registers.  The k records of every workgroup form the input of the next
// level (now with explicit indices), until one workgroup is left.  Nothing is atomic, so the
// result does not depend on scheduling.
#include "bsse_internal.h"
#include <limits.h>

namespace bsse {

namespace {

constexpr int TK_THREADS = 256;
constexpr int TK_E = 8;
constexpr int TK_SLICE = TK_THREADS * TK_E;

__device__ __forceinline__ bool tk_better(float v, long long i, float bv, long long bi)
{
    return v > bv || (v == bv && i < bi);
}

// vals[count]; idx[count] or null (then the index of element e is index_base + e).  An index of
// LLONG_MAX marks an empty record.  out_v / out_i: k records per workgroup, best first.
__global__ void __launch_bounds__(TK_THREADS)
topk_level_kernel(const float *__restrict__ vals, const long long *__restrict__ idx, long long count,
                  long long index_base, int k, float *__restrict__ out_v, long long *__restrict__ out_i)
{
    // per-wavefront winners of a round, double-buffered by round parity: one barrier per round
    __shared__ float sv[2][TK_THREADS / 64];
    __shared__ long long si[2][TK_THREADS / 64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long base = (long long)blockIdx.x * TK_SLICE;
    float v[TK_E];
    long long ix[TK_E];
    // element e of the thread sits at base + e * TK_THREADS + tid (coalesced loads)
#pragma unroll
    for (int e = 0; e < TK_E; ++e) {
        const long long pos = base + (long long)e * TK_THREADS + tid;
        const bool ok = pos < count;
        float x = ok ? vals[pos] : -INFINITY;
        if (!(x == x)) x = -INFINITY;
        v[e] = x;
        ix[e] = ok ? (idx ? idx[pos] : index_base + pos) : LLONG_MAX;
    }
    unsigned taken = 0u;
    auto rescan = [&](float &bv, long long &bi, int &be) {
        bv = -INFINITY; bi = LLONG_MAX; be = -1;
#pragma unroll
        for (int e = 0; e < TK_E; ++e) {
            if ((taken >> e) & 1u) continue;
            if (ix[e] != LLONG_MAX && (be < 0 || tk_better(v[e], ix[e], bv, bi))) { bv = v[e]; bi = ix[e]; be = e; }
        }
    };
    // (an index of LLONG_MAX is "nothing": it never beats a record and any record beats it)
    auto beats = [](float ov, long long oi, float bv, long long bi) {
        return oi != LLONG_MAX && (bi == LLONG_MAX || tk_better(ov, oi, bv, bi));
    };
    float my_v; long long my_i; int my_e;
    rescan(my_v, my_i, my_e);
    for (int r = 0; r < k; ++r) {
        float bv = my_v;
        long long bi = my_i;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const float ov = __shfl_xor(bv, d, 64);
            const long long oi = __shfl_xor(bi, d, 64);
            if (beats(ov, oi, bv, bi)) { bv = ov; bi = oi; }
        }
        const int buf = r & 1;
        if (lane == 0) { sv[buf][wave] = bv; si[buf][wave] = bi; }
        __syncthreads();
        // every thread folds the wavefronts' winners itself: no second barrier to broadcast the result
        bv = sv[buf][0]; bi = si[buf][0];
#pragma unroll
        for (int w = 1; w < TK_THREADS / 64; ++w)
            if (beats(sv[buf][w], si[buf][w], bv, bi)) { bv = sv[buf][w]; bi = si[buf][w]; }
        if (tid == 0) {
            out_v[(size_t)blockIdx.x * k + r] = bv;
            out_i[(size_t)blockIdx.x * k + r] = bi;
        }
        if (bi != LLONG_MAX && my_e >= 0 && my_i == bi) {       // indices are distinct: one owner
            taken |= 1u << my_e;
            rescan(my_v, my_i, my_e);
        }
        // (round r + 1 writes the other buffer; round r + 2 writes this one again, after everybody
        // has passed the barrier of round r + 1 and so has finished reading it)
    }
}

__global__ void gather_indexed_rows_kernel(const float *__restrict__ X, const long long *__restrict__ idx,
                                           int rows, int m, float *__restrict__ out)
{
    const int r = blockIdx.x;
    const long long c = idx[r] == LLONG_MAX ? 0 : idx[r];
    for (int i = threadIdx.x; i < m; i += blockDim.x) out[(size_t)r * m + i] = X[c * m + i];
}

}  // namespace

long long topk_level_blocks(long long count) { return (count + TK_SLICE - 1) / TK_SLICE; }

hipError_t launch_topk_level(const float *vals, const long long *idx, long long count,
                             long long index_base, int k, float *out_v, long long *out_i,
                             hipStream_t s)
{
    if (count <= 0 || k <= 0) return hipSuccess;
    hipLaunchKernelGGL(topk_level_kernel, dim3((unsigned)topk_level_blocks(count)), dim3(TK_THREADS), 0,
                       s, vals, idx, count, index_base, k, out_v, out_i);
    return hipGetLastError();
}

hipError_t launch_gather_indexed_rows(const float *X, const long long *idx, int rows, int m,
                                      float *out, hipStream_t s)
{
    if (rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(gather_indexed_rows_kernel, dim3(rows), dim3(64), 0, s, X, idx, rows, m, out);
    return hipGetLastError();
}

}  // namespace bsse
