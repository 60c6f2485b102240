// Step 5/6: grid stage of the arg-max over candidates, and the merge into the running best
// over chunks.  The sweep kernels leave one (value, global index) record per workgroup; one
// workgroup here folds them (greatest value, lowest index among equals; no float atomics, so
// the result does not depend on scheduling) and merges by the same rule (greater value, then
// lower global index), so the result does not depend on the order of the chunks either.  When the running best changes, the
// winning candidate row is copied into the handle so the chunk buffer can be recycled.
#include "bsse_internal.h"
#include <limits.h>

namespace bsse {

namespace {

constexpr int RT = 1024;

__device__ __forceinline__ bool better(float v, long long i, float bv, long long bi)
{
    return v > bv || (v == bv && i < bi);
}

__global__ void __launch_bounds__(RT)
reduce_merge_kernel(const float *__restrict__ blk_v, const long long *__restrict__ blk_i,
                    long long nblocks, const float *__restrict__ X, long long index_base, int m,
                    int first, unsigned long long *tie_counter, RunningBest *run,
                    RunningBest *run_host, float *best_x)
{
    __shared__ float sv[RT / 64];
    __shared__ long long si[RT / 64];
    __shared__ long long win;          // chunk-local row to copy, or -1

    float bv = -INFINITY;
    long long bi = LLONG_MAX;
    for (long long b = threadIdx.x; b < nblocks; b += RT) {
        const float v = blk_v[b];
        const long long i = blk_i[b];
        if (better(v, i, bv, bi)) { bv = v; bi = i; }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const float ov = __shfl_xor(bv, d, 64);
        const long long oi = __shfl_xor(bi, d, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < RT / 64; ++w)
            if (better(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; }
        long long w_row = -1;
        RunningBest r = *run;
        if (first) { r.value = 0.0f; r.has = 0; r.index = -1; r.ties = 0ull; }
        if (bi != LLONG_MAX && (!r.has || bv > r.value || (bv == r.value && bi < r.index))) {
            r.value = bv;
            r.index = bi;
            r.has = 1;
            w_row = bi - index_base;
        }
        r.ties += *tie_counter;
        *tie_counter = 0ull;                 // the next chunk starts from zero
        *run = r;
        *run_host = r;
        win = w_row;
    }
    __syncthreads();
    const long long row = win;
    if (row >= 0)
        for (int i = threadIdx.x; i < m; i += RT) best_x[i] = X[row * m + i];
}

__global__ void clear_u64_kernel(unsigned long long *p) { *p = 0ull; }

__global__ void __launch_bounds__(256) fill_zero_kernel(uint4 *p, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        p[i] = make_uint4(0u, 0u, 0u, 0u);
}

}  // namespace

// bytes must be a multiple of 16 and p 16-byte aligned
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s)
{
    if (bytes == 0) return hipSuccess;
    if (bytes % 16 != 0 || ((uintptr_t)p & 15) != 0) return hipErrorInvalidValue;
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (uint4 *)p, n16);
    return hipGetLastError();
}

hipError_t launch_clear_u64(unsigned long long *p, hipStream_t s)
{
    hipLaunchKernelGGL(clear_u64_kernel, dim3(1), dim3(1), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_reduce_merge(const float *blk_v, const long long *blk_i, long long nblocks,
                               const float *X, long long index_base, int m, int first,
                               unsigned long long *tie_counter, RunningBest *run,
                               RunningBest *run_host, float *best_x, hipStream_t s)
{
    if (nblocks <= 0) return hipSuccess;
    hipLaunchKernelGGL(reduce_merge_kernel, dim3(1), dim3(RT), 0, s, blk_v, blk_i, nblocks, X,
                       index_base, m, first, tie_counter, run, run_host, best_x);
    return hipGetLastError();
}

}  // namespace bsse
