// What this device reaches on plain kernels, measured beside the vendor peaks the roofline
// fractions are quoted against: a streaming read of a buffer far larger than the caches, a loop
// of independent matrix-core instructions (bf16 32x32x16 and fp32 32x32x2), and the latency of
// an empty launch; and the rate the bf16 matrix cores keep when a wavefront's matrix instructions
// alternate with blocks of independent vector instructions (the instruction mix of a sweep kernel
// with its loads, dependencies and barriers taken away).  Diagnostics only: nothing of the sweep
// runs here.
#include "../../include/bsse.h"
#include <hip/hip_runtime.h>
#include <chrono>
#include <cstdio>

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Every thread reads 16 bytes per trip, a wavefront 1 KiB contiguous; the sum is written only
// when it equals a value it cannot take, so the loads stay and nothing is stored.
__global__ void __launch_bounds__(256)
stream_read_kernel(const f32x4 *__restrict__ p, size_t n_vec, float *__restrict__ sink)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    f32x4 s0 = { 0, 0, 0, 0 }, s1 = { 0, 0, 0, 0 };
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + stride < n_vec; i += 2 * stride) {
        const f32x4 a = __builtin_nontemporal_load(p + i);
        const f32x4 b = __builtin_nontemporal_load(p + i + stride);
        s0 += a; s1 += b;
    }
    if (i < n_vec) s0 += __builtin_nontemporal_load(p + i);
    const float s = s0[0] + s0[1] + s0[2] + s0[3] + s1[0] + s1[1] + s1[2] + s1[3];
    if (s == -1.2345e30f) *sink = s;
}

// Eight independent accumulators per wavefront, `iters` rounds: the matrix pipe never waits for
// a result.  Operands are registers; nothing is loaded.
template <bool BF16>
__global__ void __launch_bounds__(256)
mfma_loop_kernel(int iters, float *__restrict__ sink)
{
    f32x16 acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[q][r] = 0.0f;
    const float seed = (float)(threadIdx.x & 7) * 0.125f;
    bf16x8 ab, bb;
#pragma unroll
    for (int e = 0; e < 8; ++e) { ab[e] = (__bf16)(seed + (float)e); bb[e] = (__bf16)(1.0f - seed); }
    const float af = seed + 1.0f, bf = 2.0f - seed;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            if constexpr (BF16) acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab, bb, acc[q], 0, 0, 0);
            else acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(af, bf, acc[q], 0, 0, 0);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[q][r];
    if (s == -1.2345e30f) *sink = s;
}

__global__ void empty_kernel() {}

// Rounds of `mfma_groups` x 4 matrix instructions (four independent accumulators) followed by
// `valu_groups` x 24 vector instructions of the kinds an arg-max epilogue is made of (three-operand
// maximum, compare into a scalar mask, select under a scalar mask, in equal parts, two
// independent chains), eight wavefronts per workgroup and one workgroup per compute unit (the
// dynamic LDS the launch asks for keeps a second one away): two wavefronts per SIMD, each with
// the other's vector block to run beside its matrix block.  Nothing is loaded or stored.
#define BSSE_MIX6                                                                             \
    "v_max3_f32 %[v0], %[v0], %[c0], %[c1]\n\t"                                               \
    "v_max3_f32 %[v1], %[v1], %[c1], %[c0]\n\t"                                               \
    "v_cmp_eq_f32 %[m0], %[v0], %[c0]\n\t"                                                    \
    "v_cmp_eq_f32 %[m1], %[v1], %[c0]\n\t"                                                    \
    "s_nop 0\n\t"                                                                             \
    "v_cndmask_b32 %[w0], %[w0], %[c1], %[m0]\n\t"                                            \
    "v_cndmask_b32 %[w1], %[w1], %[c0], %[m1]\n\t"
__global__ void __launch_bounds__(512, 2)
mixed_loop_kernel(int rounds, int mfma_groups, int valu_groups, float *__restrict__ sink)
{
    f32x16 acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[q][r] = 0.0f;
    const float seed = (float)(threadIdx.x & 7) * 0.125f;
    bf16x8 ab, bb;
#pragma unroll
    for (int e = 0; e < 8; ++e) { ab[e] = (__bf16)(seed + (float)e); bb[e] = (__bf16)(1.0f - seed); }
    float v0 = seed, v1 = seed + 1.0f, w0 = 0.0f, w1 = 0.0f;
    const float c0 = 0.5f + seed, c1 = 0.25f;
    // (long trips first, the remainder in short ones: the loop overhead of a short trip is a few
    // per cent of its instructions' issue time)
    auto mfma4 = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab, bb, acc[q], 0, 0, 0);
    };
    auto valu24 = [&]() __attribute__((always_inline)) {
        unsigned long long m0, m1;
        asm volatile(BSSE_MIX6 BSSE_MIX6 BSSE_MIX6 BSSE_MIX6
                     : [v0] "+v"(v0), [v1] "+v"(v1), [w0] "+v"(w0), [w1] "+v"(w1), [m0] "=&s"(m0), [m1] "=&s"(m1)
                     : [c0] "v"(c0), [c1] "v"(c1));
    };
#pragma unroll 1
    for (int it = 0; it < rounds; ++it) {
#pragma unroll 1
        for (int g = 0; g < (mfma_groups >> 3); ++g) {
#pragma unroll
            for (int e = 0; e < 8; ++e) mfma4();
        }
#pragma unroll 1
        for (int g = 0; g < (mfma_groups & 7); ++g) mfma4();
#pragma unroll 1
        for (int g = 0; g < (valu_groups >> 2); ++g) {
            valu24(); valu24(); valu24(); valu24();
        }
#pragma unroll 1
        for (int g = 0; g < (valu_groups & 3); ++g) valu24();
    }
    float s = v0 + v1 + w0 + w1;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[q][r];
    if (s == -1.2345e30f) *sink = s;
}

struct Ev {
    hipEvent_t a = nullptr, b = nullptr;
    ~Ev() { if (a) (void)hipEventDestroy(a); if (b) (void)hipEventDestroy(b); }
};

}  // namespace

#define CEIL_TRY(call)                                                                        \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) {                                                               \
            if (buf) (void)hipFree(buf);                                                      \
            if (sink) (void)hipFree(sink);                                                    \
            if (prev >= 0) (void)hipSetDevice(prev);                                          \
            return e_ == hipErrorOutOfMemory ? BSSE_ENOMEM : BSSE_EDEVICE;                    \
        }                                                                                     \
    } while (0)

extern "C" bsse_status bsse_measure_ceilings(int device, double *stream_read_gbs, double *mfma_bf16_tflops,
                                             double *mfma_f32_tflops, double *empty_launch_us)
{
    if (!stream_read_gbs || !mfma_bf16_tflops || !mfma_f32_tflops || !empty_launch_us) return BSSE_EINVAL;
    if (device < -1) return BSSE_EINVAL;
    void *buf = nullptr;
    float *sink = nullptr;
    int prev = -1;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return BSSE_EDEVICE;
    if (device >= ndev) return BSSE_EINVAL;
    if (device >= 0) {
        int cur = -1;
        if (hipGetDevice(&cur) != hipSuccess) return BSSE_EDEVICE;
        if (cur != device) { prev = cur; if (hipSetDevice(device) != hipSuccess) return BSSE_EDEVICE; }
    }
    int dev = device;
    if (dev < 0) CEIL_TRY(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    CEIL_TRY(hipGetDeviceProperties(&prop, dev));
    const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    Ev ev;
    CEIL_TRY(hipEventCreate(&ev.a));
    CEIL_TRY(hipEventCreate(&ev.b));
    CEIL_TRY(hipMalloc((void **)&sink, 256));

    // ---- streaming read: 2 GiB, eight times the last-level cache
    const size_t bytes = (size_t)2 << 30, n_vec = bytes / 16;
    CEIL_TRY(hipMalloc(&buf, bytes));
    CEIL_TRY(hipMemset(buf, 0, bytes));
    double best_ms = 1e30;
    for (int rep = 0; rep < 6; ++rep) {
        CEIL_TRY(hipEventRecord(ev.a, nullptr));
        hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)(cus * 8)), dim3(256), 0, nullptr,
                           (const f32x4 *)buf, n_vec, sink);
        CEIL_TRY(hipGetLastError());
        CEIL_TRY(hipEventRecord(ev.b, nullptr));
        CEIL_TRY(hipEventSynchronize(ev.b));
        float ms = 0.0f;
        CEIL_TRY(hipEventElapsedTime(&ms, ev.a, ev.b));
        if (rep > 0 && ms < best_ms) best_ms = ms;
    }
    const double read_gbs = (double)bytes / (best_ms * 1e-3) / 1e9;
    (void)hipFree(buf);
    buf = nullptr;

    // ---- matrix-core loops: two workgroups of four wavefronts per compute unit
    double tf[2] = { 0.0, 0.0 };
    for (int pass = 0; pass < 2; ++pass) {
        const int iters = pass == 0 ? 4096 : 1024;
        const double flops_per_mfma = pass == 0 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
        const unsigned blocks = (unsigned)(cus * 2);
        double best = 1e30;
        for (int rep = 0; rep < 4; ++rep) {
            CEIL_TRY(hipEventRecord(ev.a, nullptr));
            if (pass == 0) hipLaunchKernelGGL(mfma_loop_kernel<true>, dim3(blocks), dim3(256), 0, nullptr, iters, sink);
            else hipLaunchKernelGGL(mfma_loop_kernel<false>, dim3(blocks), dim3(256), 0, nullptr, iters, sink);
            CEIL_TRY(hipGetLastError());
            CEIL_TRY(hipEventRecord(ev.b, nullptr));
            CEIL_TRY(hipEventSynchronize(ev.b));
            float ms = 0.0f;
            CEIL_TRY(hipEventElapsedTime(&ms, ev.a, ev.b));
            if (rep > 0 && ms < best) best = ms;
        }
        const double total = (double)blocks * 4.0 * iters * 8.0 * flops_per_mfma;
        tf[pass] = total / (best * 1e-3) / 1e12;
    }

    // ---- empty launches back to back, waited for once: time per launch
    for (int q = 0; q < 20; ++q) hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, nullptr);
    CEIL_TRY(hipDeviceSynchronize());
    const int n = 2000;
    const auto t0 = std::chrono::steady_clock::now();
    for (int q = 0; q < n; ++q) hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, nullptr);
    CEIL_TRY(hipDeviceSynchronize());
    const auto t1 = std::chrono::steady_clock::now();
    *empty_launch_us = std::chrono::duration<double, std::micro>(t1 - t0).count() / n;
    *stream_read_gbs = read_gbs; *mfma_bf16_tflops = tf[0]; *mfma_f32_tflops = tf[1];

    (void)hipFree(sink);
    if (prev >= 0) (void)hipSetDevice(prev);
    return BSSE_OK;
}

#define MIX_TRY(call)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) {                                                               \
            if (sink) (void)hipFree(sink);                                                    \
            if (prev >= 0) (void)hipSetDevice(prev);                                          \
            return e_ == hipErrorOutOfMemory ? BSSE_ENOMEM : BSSE_EDEVICE;                    \
        }                                                                                     \
    } while (0)

extern "C" bsse_status bsse_measure_mixed_ceiling(int device, int mfma_per_round, int valu_per_round,
                                                  double *mfma_bf16_tflops)
{
    if (!mfma_bf16_tflops || device < -1) return BSSE_EINVAL;
    if (mfma_per_round < 4 || mfma_per_round > 4096 || mfma_per_round % 4 != 0) return BSSE_EINVAL;
    if (valu_per_round < 0 || valu_per_round > 65536 || valu_per_round % 24 != 0) return BSSE_EINVAL;
    float *sink = nullptr;
    int prev = -1;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return BSSE_EDEVICE;
    if (device >= ndev) return BSSE_EINVAL;
    if (device >= 0) {
        int cur = -1;
        if (hipGetDevice(&cur) != hipSuccess) return BSSE_EDEVICE;
        if (cur != device) { prev = cur; if (hipSetDevice(device) != hipSuccess) return BSSE_EDEVICE; }
    }
    int dev = device;
    if (dev < 0) MIX_TRY(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    MIX_TRY(hipGetDeviceProperties(&prop, dev));
    const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    Ev ev;
    MIX_TRY(hipEventCreate(&ev.a));
    MIX_TRY(hipEventCreate(&ev.b));
    MIX_TRY(hipMalloc((void **)&sink, 256));
    const int lds = 96 * 1024;                 // more than half of a compute unit's LDS: one workgroup each
    MIX_TRY(hipFuncSetAttribute((const void *)mixed_loop_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    // about 2e5 matrix instructions per wavefront: tens of milliseconds
    const int rounds = 200000 / mfma_per_round > 0 ? 200000 / mfma_per_round : 1;
    double best = 1e30;
    for (int rep = 0; rep < 4; ++rep) {
        MIX_TRY(hipEventRecord(ev.a, nullptr));
        hipLaunchKernelGGL(mixed_loop_kernel, dim3((unsigned)cus), dim3(512), (size_t)lds, nullptr, rounds,
                           mfma_per_round / 4, valu_per_round / 24, sink);
        MIX_TRY(hipGetLastError());
        MIX_TRY(hipEventRecord(ev.b, nullptr));
        MIX_TRY(hipEventSynchronize(ev.b));
        float ms = 0.0f;
        MIX_TRY(hipEventElapsedTime(&ms, ev.a, ev.b));
        if (rep > 0 && ms < best) best = ms;
    }
    const double total = (double)cus * 8.0 * rounds * mfma_per_round * (2.0 * 32 * 32 * 16);
    *mfma_bf16_tflops = total / (best * 1e-3) / 1e12;
    (void)hipFree(sink);
    if (prev >= 0) (void)hipSetDevice(prev);
    return BSSE_OK;
}
