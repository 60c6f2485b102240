// libbsse C ABI: argument checking, payoff packing, device bookkeeping and the chunked sweep
// driver.  Everything numeric happens in the kernels; nothing here evaluates a payoff.
#include "../../include/bsse.h"
#include "bsse_internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <algorithm>
#include <mutex>
#include <vector>

using namespace bsse;

// ------------------------------------------------------------------------------ errors
static thread_local char g_err[320] = "";

static bsse_status fail(bsse_status s, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return s;
}

extern "C" const char *bsse_last_error(void) { return g_err; }

extern "C" const char *bsse_status_name(bsse_status s)
{
    // (a C caller can hand over any integer: read it as one)
    int code;
    memcpy(&code, &s, sizeof(code));
    static_assert(sizeof(code) == sizeof(s), "status codes are ints");
    switch (code) {
    case BSSE_OK: return "BSSE_OK";
    case BSSE_EINVAL: return "BSSE_EINVAL";
    case BSSE_ENOTFINITE: return "BSSE_ENOTFINITE";
    case BSSE_EOVERFLOW: return "BSSE_EOVERFLOW";
    case BSSE_ENOMEM: return "BSSE_ENOMEM";
    case BSSE_EDEVICE: return "BSSE_EDEVICE";
    case BSSE_ESTATE: return "BSSE_ESTATE";
    }
    return "BSSE_?";
}

#define HIP_TRY(call)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail(e_ == hipErrorOutOfMemory ? BSSE_ENOMEM : BSSE_EDEVICE, "%s: %s",     \
                        #call, hipGetErrorString(e_));                                        \
    } while (0)

// ------------------------------------------------------------------------------ handle
struct HostOut {            // pinned, device-visible: kernels write results here directly
    RunningBest run;        // by the merge kernel of every chunk
    float fin_v;            // by the one-row re-evaluation of the winner
};

// Device scratch of the prior batch: kept by the handle and grown on demand, so that repeated
// calls do not allocate.
struct PriorScratch {
    float *L = nullptr, *priors = nullptr, *blk_v = nullptr, *rows = nullptr;
    long long *blk_i = nullptr;
    bsse::PriorBest *run = nullptr;
    int32_t *br = nullptr;
    unsigned long long *ties = nullptr;
    size_t cap_L = 0, cap_priors = 0, cap_blk_v = 0, cap_rows = 0, cap_blk_i = 0, cap_run = 0,
           cap_br = 0, cap_ties = 0;
    unsigned char *host = nullptr;   // pinned staging: priors on the way in, results on the way out
    size_t cap_host = 0;
    void release()
    {
        if (host) (void)hipHostFree(host);
        (void)hipFree(L); (void)hipFree(priors); (void)hipFree(blk_v); (void)hipFree(rows);
        (void)hipFree(blk_i); (void)hipFree(run); (void)hipFree(br); (void)hipFree(ties);
    }
};

// Device scratch of the top-k entry point: kept by the handle and grown on demand.
struct TopkScratch {
    void *p[9] = { nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr };
    size_t cap[9] = { 0, 0, 0, 0, 0, 0, 0, 0, 0 };
    void release() { for (void *q : p) (void)hipFree(q); }
};

// Device scratch of the streamed sweep: one record per workgroup of a chunk, the running best, the
// winning row, the tie counter, the per-type leader payoffs of the re-evaluated winner and (small-
// game kernel) the workgroups' running-best slots.  Owned by the handle and grown on demand, or
// (`fixed`) a carving of the library's static scratch array that cannot grow.
struct Work {
    float *blk_v = nullptr;
    long long *blk_i = nullptr;
    long long blk_cap = 0;
    SmallSlot *slots = nullptr;      // slot_sets sets of small_num_slots() slots
    int slot_sets = 0;
    RunningBest *run = nullptr;
    float *best_x = nullptr;
    unsigned long long *tie_counter = nullptr;
    float *win_l = nullptr;          // [K]
    bool fixed = false;
};

struct bsse_game {
    int m = 0, n = 0, K = 0, storage = 0, device = 0;
    PathKind path = PATH_VALU;
    hipStream_t stream = nullptr;
    GameView view{};
    // device allocations
    float *dB = nullptr, *dAT = nullptr, *dprior = nullptr;
    void *dBpack = nullptr, *dATpack = nullptr;
    float *gen = nullptr;
    long long gen_count = -1;
    size_t gen_cap = 0;
    unsigned long long *lat_table = nullptr;
    size_t lat_table_cap = 0;
    int lat_table_N = -1;        // resolution the table on the device was built for (-1: none)
    Work w;                      // the scratch in use
    // small-game kernel: per-workgroup running bests of the current sweep, folded on demand
    unsigned epoch = 0;          // of the current sweep (slots of other epochs are stale)
    bool fold_pending = false;   // chunks swept since the last fold
    bool fold_first = true;      // the next fold is the first of its sweep
    bool ties_dirty = false;     // the device tie counter may be non-zero
    // Chunks of generated rows need no input from the caller's stream, so after the first chunk of
    // a sweep they alternate between two streams of the handle's own (slot sets 0 and 1; chunks on
    // the caller's stream use set 2): the end of one launch then overlaps the start of the next.
    // Events order them behind the caller's stream (fork) and the fold behind them (join).
    hipStream_t aux[2] = { nullptr, nullptr };
    hipEvent_t aux_fork = nullptr, aux_join[2] = { nullptr, nullptr };
    bool aux_used[2] = { false, false };           // work enqueued since the last join
    unsigned chunk_seq = 0;                        // chunks of the current sweep
    PriorScratch pri;
    TopkScratch topk;
    // host copies of the game as given to create (fp32, unrounded): the profile LP of bsse_polish
    std::vector<float> hA, hB, hprior;
    float *stage = nullptr;                        // generated rows on their way into a sweep
    size_t stage_cap = 0;
    float *centre_dev = nullptr;                   // [m] centre of a local candidate set
    float *pol_rows = nullptr, *pol_v = nullptr;   // device scratch of bsse_polish
    int32_t *pol_br = nullptr;
    // pinned host
    HostOut *h_out = nullptr;
    int32_t *h_br = nullptr;
    long long n_evals = 0;
    bool fresh = true;       // the next chunk starts a new sweep
    bool result_valid = false;   // bsse_sweep_result has reported the sweep in the handle's own scratch
    // kernel timing
    bool timing = false;
    std::vector<hipEvent_t> ev;      // start/stop pairs of recorded launches
    std::vector<hipEvent_t> ev_pool; // recycled events
    double timed_ms = 0.0;
    long long timed_launches = 0;
};

namespace {

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) prev = -1;
        ok = (prev == dev) || hipSetDevice(dev) == hipSuccess;
        if (prev == dev) prev = -1;
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

float host_round_bf16(float v)
{
    uint32_t b;
    memcpy(&b, &v, 4);
    b += 0x7FFFu + ((b >> 16) & 1u);
    b &= 0xFFFF0000u;
    memcpy(&v, &b, 4);
    return v;
}

// C(N+m-1, m-1) with overflow detection; returns false when it exceeds `cap`.
bool lattice_count_checked(int m, int N, unsigned long long cap, unsigned long long *out)
{
    unsigned long long k = (unsigned long long)(m - 1), a = (unsigned long long)N + k;
    if (k > (unsigned long long)N) k = (unsigned long long)N;       // C(a,k) = C(a,a-k)
    unsigned __int128 c = 1;
    for (unsigned long long i = 1; i <= k; ++i) {
        c = c * (a - k + i) / i;             // exact: a product of i consecutive integers / i!
        if (c > (unsigned __int128)cap) return false;
    }
    *out = (unsigned long long)c;
    return true;
}

constexpr unsigned long long LATTICE_MAX = 1ull << 40;
constexpr long long CHUNK_MAX = 1ll << 31;

void free_game(bsse_game *g)
{
    if (!g) return;
    DeviceGuard dg(g->device);
    (void)hipFree(g->dB); (void)hipFree(g->dAT); (void)hipFree(g->dprior);
    (void)hipFree(g->dBpack); (void)hipFree(g->dATpack);
    (void)hipFree(g->gen); (void)hipFree(g->lat_table);
    (void)hipFree(g->w.blk_v); (void)hipFree(g->w.blk_i); (void)hipFree(g->w.slots);
    (void)hipFree(g->w.run); (void)hipFree(g->w.best_x); (void)hipFree(g->w.tie_counter);
    (void)hipFree(g->w.win_l);
    g->pri.release();
    g->topk.release();
    (void)hipFree(g->pol_rows); (void)hipFree(g->pol_v); (void)hipFree(g->pol_br);
    for (int q = 0; q < 2; ++q) {
        if (g->aux[q]) { (void)hipStreamSynchronize(g->aux[q]); (void)hipStreamDestroy(g->aux[q]); }
        if (g->aux_join[q]) (void)hipEventDestroy(g->aux_join[q]);
    }
    if (g->aux_fork) (void)hipEventDestroy(g->aux_fork);
    (void)hipFree(g->centre_dev); (void)hipFree(g->stage);
    if (g->h_out) (void)hipHostFree(g->h_out);
    if (g->h_br) (void)hipHostFree(g->h_br);
    for (hipEvent_t e : g->ev) (void)hipEventDestroy(e);
    for (hipEvent_t e : g->ev_pool) (void)hipEventDestroy(e);
    delete g;
}

bsse_status ensure_blocks(bsse_game *g, long long nblocks)
{
    if (nblocks <= g->w.blk_cap) return BSSE_OK;
    if (g->w.fixed)
        return fail(BSSE_EOVERFLOW, "%lld workgroup records exceed the %lld the static scratch holds",
                    nblocks, g->w.blk_cap);
    // the stream may still be reading the old workspace
    HIP_TRY(hipStreamSynchronize(g->stream));
    (void)hipFree(g->w.blk_v); (void)hipFree(g->w.blk_i);
    g->w.blk_v = nullptr; g->w.blk_i = nullptr; g->w.blk_cap = 0;
    HIP_TRY(hipMalloc((void **)&g->w.blk_v, (size_t)nblocks * sizeof(float)));
    HIP_TRY(hipMalloc((void **)&g->w.blk_i, (size_t)nblocks * sizeof(long long)));
    g->w.blk_cap = nblocks;
    return BSSE_OK;
}

bsse_status ensure_gen(bsse_game *g, unsigned long long rows)
{
    const unsigned long long bytes = rows * (unsigned long long)g->m * sizeof(float);
    if (bytes <= g->gen_cap) return BSSE_OK;
    HIP_TRY(hipStreamSynchronize(g->stream));
    (void)hipFree(g->gen);
    g->gen = nullptr; g->gen_cap = 0; g->gen_count = -1;
    size_t free_b = 0, total_b = 0;
    HIP_TRY(hipMemGetInfo(&free_b, &total_b));
    if (bytes > free_b)
        return fail(BSSE_EOVERFLOW, "candidate buffer of %llu bytes exceeds free device memory (%zu)",
                    bytes, free_b);
    HIP_TRY(hipMalloc((void **)&g->gen, (size_t)bytes));
    g->gen_cap = (size_t)bytes;
    return BSSE_OK;
}

hipError_t launch_sweep_on(bsse_game *g, const SweepArgs &a, bool eval, hipStream_t stream)
{
    if (g->path == PATH_VALU) return launch_sweep_valu(g->view, a, eval, stream);
    (void)eval;
    return launch_sweep_mfma(g->view, a, stream);
}

hipError_t launch_sweep(bsse_game *g, const SweepArgs &a, bool eval)
{
    return launch_sweep_on(g, a, eval, g->stream);
}

long long sweep_blocks(const bsse_game *g, long long count)
{
    return g->path == PATH_VALU ? valu_num_blocks(count) : mfma_num_blocks(g->view.variant, count);
}

bsse_status take_event(bsse_game *g, hipEvent_t *e)
{
    if (!g->ev_pool.empty()) { *e = g->ev_pool.back(); g->ev_pool.pop_back(); return BSSE_OK; }
    HIP_TRY(hipEventCreate(e));
    return BSSE_OK;
}

// Wait for everything the handle has enqueued, on the caller's stream and on its own.
bsse_status sync_all(bsse_game *g)
{
    for (int q = 0; q < 2; ++q)
        if (g->aux[q]) { HIP_TRY(hipStreamSynchronize(g->aux[q])); g->aux_used[q] = false; }
    HIP_TRY(hipStreamSynchronize(g->stream));
    return BSSE_OK;
}

bsse_status drain_timing(bsse_game *g)
{
    for (size_t i = 0; i + 1 < g->ev.size(); i += 2) {
        float ms = 0.0f;
        HIP_TRY(hipEventElapsedTime(&ms, g->ev[i], g->ev[i + 1]));
        g->timed_ms += ms;
        g->timed_launches += 1;
    }
    for (hipEvent_t e : g->ev) g->ev_pool.push_back(e);
    g->ev.clear();
    return BSSE_OK;
}

}  // namespace

// ---------------------------------------------------------------------- static scratch
// Scratch of bsse_sweep_static: a file-scope device array, so that the entry point allocates
// nothing.  Every GPU the library runs on holds its own copy (1.2 MiB) until the process ends; the
// array's name is only a host-side stand-in, the device address is looked up once per device with
// hipGetSymbolAddress and that pointer is what kernels and fills are given.
namespace {

constexpr long long STATIC_MAX_BLOCKS = 65536;    // workgroup records of one chunk
constexpr int STATIC_MAX_M = 4096, STATIC_MAX_K = 65536, STATIC_MAX_SLOTS = 2048;
constexpr size_t ST_OFF_RUN = 0, ST_OFF_TIES = 256, ST_OFF_BESTX = 512,
                 ST_OFF_WINL = ST_OFF_BESTX + (size_t)STATIC_MAX_M * sizeof(float),
                 ST_OFF_BLKV = ST_OFF_WINL + (size_t)STATIC_MAX_K * sizeof(float),
                 ST_OFF_BLKI = ST_OFF_BLKV + (size_t)STATIC_MAX_BLOCKS * sizeof(float),
                 ST_OFF_SLOTS = ST_OFF_BLKI + (size_t)STATIC_MAX_BLOCKS * sizeof(long long),
                 STATIC_BYTES = ST_OFF_SLOTS + (size_t)STATIC_MAX_SLOTS * sizeof(SmallSlot);
static_assert(sizeof(RunningBest) <= 256 && sizeof(SmallSlot) == 64, "scratch layout");
static_assert(ST_OFF_WINL % 256 == 0 && ST_OFF_BLKV % 256 == 0 && ST_OFF_BLKI % 256 == 0 &&
              ST_OFF_SLOTS % 256 == 0, "scratch parts stay 256-byte aligned");

}  // namespace

static __device__ __align__(256) unsigned char scratch[STATIC_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
unsigned char *g_scratch_ptr[MAX_DEVICES];      // per device: the address of its copy of `scratch`
std::mutex g_scratch_mutex;

// With device `dev` current: the device address of that device's scratch array (looked up on the
// first call per device).
bsse_status static_scratch(int dev, unsigned char **out)
{
    if (dev < 0 || dev >= MAX_DEVICES) return fail(BSSE_EDEVICE, "device ordinal %d is beyond %d", dev, MAX_DEVICES - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(BSSE_EDEVICE, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
    }
    *out = g_scratch_ptr[dev];
    return BSSE_OK;
}

}  // namespace

// ------------------------------------------------------------------------------ create
extern "C" bsse_status bsse_create(int m, int n, int K, const float *A, const float *B,
                                   const float *prior, bsse_game **out)
{
    bsse_options opt = { BSSE_STORAGE_F32, BSSE_PATH_AUTO, -1 };
    return bsse_create_ex(m, n, K, A, B, prior, &opt, out);
}

extern "C" bsse_status bsse_create_ex(int m, int n, int K, const float *A, const float *B,
                                      const float *prior, const bsse_options *opt,
                                      bsse_game **out)
{
    g_err[0] = 0;
    if (!out) return fail(BSSE_EINVAL, "out is NULL");
    if (!A || !B || !prior) return fail(BSSE_EINVAL, "A, B and prior must not be NULL");
    if (!opt) return fail(BSSE_EINVAL, "opt is NULL");
    if (m < 1 || n < 1 || K < 1) return fail(BSSE_EINVAL, "m, n, K must be >= 1 (got %d, %d, %d)", m, n, K);
    if (m > 4096 || n > 65535 || K > 65535)
        return fail(BSSE_EINVAL, "limits: m <= 4096, n <= 65535, K <= 65535 (got %d, %d, %d)", m, n, K);
    const unsigned long long elems = (unsigned long long)m * n * K;
    if (elems > (1ull << 28)) return fail(BSSE_EINVAL, "K*m*n = %llu exceeds 2^28", elems);
    if (opt->storage != BSSE_STORAGE_F32 && opt->storage != BSSE_STORAGE_BF16)
        return fail(BSSE_EINVAL, "unknown storage option %d", opt->storage);
    if (opt->path != BSSE_PATH_AUTO && opt->path != BSSE_PATH_VALU && opt->path != BSSE_PATH_MFMA &&
        opt->path != BSSE_PATH_MFMA_SPLIT)
        return fail(BSSE_EINVAL, "unknown path option %d", opt->path);
    if (opt->device < -1) return fail(BSSE_EINVAL, "bad device ordinal %d", opt->device);
    for (unsigned long long e = 0; e < elems; ++e)
        if (!std::isfinite(A[e]) || !std::isfinite(B[e]))
            return fail(BSSE_ENOTFINITE, "payoff entry %llu is not finite", e);
    double psum = 0.0;
    for (int t = 0; t < K; ++t) {
        if (!std::isfinite(prior[t])) return fail(BSSE_ENOTFINITE, "prior[%d] is not finite", t);
        if (prior[t] < 0.0f) return fail(BSSE_EINVAL, "prior[%d] is negative", t);
        psum += (double)prior[t];
    }
    if (std::fabs(psum - 1.0) > 1e-6) return fail(BSSE_EINVAL, "prior sums to %.9g, not 1", psum);
    // which kernel family: the small-game kernel, the split path, plain MFMA, else VALU
    const bool bf = opt->storage == BSSE_STORAGE_BF16;
    bool exact = true;                       // every payoff is a bf16 number
    for (unsigned long long e = 0; e < elems && exact; ++e)
        exact = host_round_bf16(A[e]) == A[e] && host_round_bf16(B[e]) == B[e];
    int variant = -1;
    PathKind path = PATH_VALU;
    if (opt->path == BSSE_PATH_MFMA_SPLIT) {
        if (bf) return fail(BSSE_EINVAL, "the split path takes fp32 storage");
        variant = mfma_select(m, n, K, 2, exact);
        if (variant < 0) return fail(BSSE_EINVAL, "shape m=%d n=%d K=%d has no split MFMA path", m, n, K);
        path = PATH_MFMA_SPLIT;
    } else if (opt->path == BSSE_PATH_MFMA) {
        variant = mfma_select(m, n, K, bf ? 1 : 0, exact);
        if (variant < 0) return fail(BSSE_EINVAL, "shape m=%d n=%d K=%d has no MFMA path", m, n, K);
        path = bf ? PATH_MFMA_BF16 : PATH_MFMA_F32;
    } else if (opt->path == BSSE_PATH_AUTO) {
        if (bf) {
            variant = mfma_select(m, n, K, 1, exact);
            if (variant >= 0) path = PATH_MFMA_BF16;
        } else {
            if (small_supported(m, n, K, 0)) {
                variant = mfma_select(m, n, K, 0, exact);
                path = PATH_MFMA_F32;
            } else if ((variant = mfma_select(m, n, K, 2, exact)) >= 0) {
                path = PATH_MFMA_SPLIT;
            } else if ((variant = mfma_select(m, n, K, 0, exact)) >= 0) {
                path = PATH_MFMA_F32;
            }
        }
    }
    const bool use_mfma = path != PATH_VALU;

    // ---- device
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1)
        return fail(BSSE_EDEVICE, "no HIP device is visible");
    int dev = opt->device;
    if (dev < 0 && hipGetDevice(&dev) != hipSuccess) return fail(BSSE_EDEVICE, "hipGetDevice failed");
    if (dev >= ndev) return fail(BSSE_EINVAL, "device %d of %d does not exist", dev, ndev);
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(BSSE_EDEVICE, "device %d is %s; this library holds gfx950 code only", dev,
                    prop.gcnArchName);

    bsse_game *g = new (std::nothrow) bsse_game;
    if (!g) return fail(BSSE_ENOMEM, "host allocation failed");
    g->m = m; g->n = n; g->K = K; g->storage = opt->storage; g->device = dev;
    g->path = path;
    try {
        g->hA.assign(A, A + elems); g->hB.assign(B, B + elems); g->hprior.assign(prior, prior + K);
    } catch (...) { delete g; return fail(BSSE_ENOMEM, "host allocation failed"); }
    g->view.variant = variant;

    DeviceGuard dg(dev);
    if (!dg.ok) { free_game(g); return fail(BSSE_EDEVICE, "hipSetDevice(%d) failed", dev); }

    // ---- pack on the host: optional bf16 rounding, B as given, A transposed per type
    std::vector<float> hB(elems), hAT(elems), hA;
    for (unsigned long long e = 0; e < elems; ++e) hB[e] = bf ? host_round_bf16(B[e]) : B[e];
    for (int t = 0; t < K; ++t)
        for (int i = 0; i < m; ++i)
            for (int j = 0; j < n; ++j) {
                const float a = A[((size_t)t * m + i) * n + j];
                hAT[((size_t)t * n + j) * m + i] = bf ? host_round_bf16(a) : a;
            }

    bsse_status st = BSSE_OK;
    auto up = [&](void **dst, const void *src, size_t bytes) -> bsse_status {
        HIP_TRY(hipMalloc(dst, bytes));
        HIP_TRY(hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice));
        return BSSE_OK;
    };
    auto zeroed = [&](void **dst, size_t bytes) -> bsse_status {
        HIP_TRY(hipMalloc(dst, bytes));
        HIP_TRY(hipMemset(*dst, 0, bytes));
        return BSSE_OK;
    };
    do {
        if ((st = up((void **)&g->dB, hB.data(), elems * 4)) != BSSE_OK) break;
        if ((st = up((void **)&g->dAT, hAT.data(), elems * 4)) != BSSE_OK) break;
        if ((st = up((void **)&g->dprior, prior, (size_t)K * 4)) != BSSE_OK) break;
        g->view.m_pad = m; g->view.n_pad = n;
        if (use_mfma) {
            void *pb = nullptr, *pa = nullptr;
            size_t bb = 0, ab = 0;
            mfma_pack(variant, m, n, K, A, B, &pb, &bb, &pa, &ab, &g->view.m_pad, &g->view.n_pad);
            if (!pb || !pa) { free(pb); free(pa); st = fail(BSSE_ENOMEM, "host allocation failed"); break; }
            st = up(&g->dBpack, pb, bb);
            if (st == BSSE_OK) st = up(&g->dATpack, pa, ab);
            free(pb); free(pa);
            if (st != BSSE_OK) break;
            hipError_t pe = mfma_prepare(variant, K);
            if (pe != hipSuccess) { st = fail(BSSE_EDEVICE, "mfma_prepare: %s", hipGetErrorString(pe)); break; }
        }
        if ((st = zeroed((void **)&g->w.run, sizeof(RunningBest))) != BSSE_OK) break;
        if ((st = zeroed((void **)&g->w.best_x, (size_t)m * 4)) != BSSE_OK) break;
        if ((st = zeroed((void **)&g->w.tie_counter, 8)) != BSSE_OK) break;
        if (use_mfma && mfma_is_small(variant) &&       // epoch 0 marks a slot never written
            (st = zeroed((void **)&g->w.slots, (size_t)3 * small_num_slots() * sizeof(SmallSlot))) != BSSE_OK) break;
        g->w.slot_sets = g->w.slots ? 3 : 0;
        if ((st = zeroed((void **)&g->w.win_l, (size_t)K * 4)) != BSSE_OK) break;
        hipError_t e = hipHostMalloc((void **)&g->h_out, sizeof(HostOut), hipHostMallocDefault);
        if (e == hipSuccess) e = hipHostMalloc((void **)&g->h_br, (size_t)K * 4, hipHostMallocDefault);
        if (e != hipSuccess) { st = fail(BSSE_ENOMEM, "hipHostMalloc: %s", hipGetErrorString(e)); break; }
    } while (0);
    if (st != BSSE_OK) { free_game(g); return st; }

    {   // set-up of the static scratch for this device (bsse_sweep_static reports a failure itself)
        unsigned char *unused = nullptr;
        (void)static_scratch(dev, &unused);
        g_err[0] = 0;
    }
    g->view.m = m; g->view.n = n; g->view.K = K;
    g->view.x_bf16 = bf ? 1 : 0;
    g->view.B = g->dB; g->view.AT = g->dAT; g->view.prior = g->dprior;
    g->view.Bpack = g->dBpack; g->view.ATpack = g->dATpack;
    *out = g;
    return BSSE_OK;
}

extern "C" void bsse_destroy(bsse_game *g)
{
    if (!g) return;
    {
        DeviceGuard dg(g->device);
        (void)sync_all(g);
    }
    free_game(g);
}

extern "C" bsse_status bsse_set_stream(bsse_game *g, void *hip_stream)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    DeviceGuard dg(g->device);
    bsse_status st = sync_all(g);                 // earlier work keeps its order
    if (st != BSSE_OK) return st;
    g->stream = (hipStream_t)hip_stream;
    return BSSE_OK;
}

extern "C" const char *bsse_path_name(const bsse_game *g)
{
    if (!g) return "";
    switch (g->path) {
    case PATH_VALU: return g->storage == BSSE_STORAGE_BF16 ? "valu_bf16" : "valu";
    case PATH_MFMA_F32:
    case PATH_MFMA_BF16:
    case PATH_MFMA_SPLIT: return mfma_variant_name(g->view.variant);
    }
    return "";
}

// --------------------------------------------------------------------------- generation
extern "C" bsse_status bsse_lattice_count(int m, int N, int64_t *count_out)
{
    g_err[0] = 0;
    if (!count_out) return fail(BSSE_EINVAL, "count_out is NULL");
    if (m < 1 || m > 4096) return fail(BSSE_EINVAL, "m must be in 1..4096 (got %d)", m);
    if (N < 1 || N > (1 << 24)) return fail(BSSE_EINVAL, "N must be in 1..2^24 (got %d)", N);
    unsigned long long c = 0;
    if (!lattice_count_checked(m, N, LATTICE_MAX, &c))
        return fail(BSSE_EOVERFLOW, "lattice of resolution %d in %d parts has more than 2^40 points", N, m);
    *count_out = (int64_t)c;
    return BSSE_OK;
}

namespace {

// centre (host [m]) and radius of a local set: validated, the centre uploaded to the handle
bsse_status check_around(const bsse_game *g, const float *centre, float radius)
{
    if (!centre) return fail(BSSE_EINVAL, "centre is NULL");
    if (!(radius >= 0.0f && radius <= 1.0f)) return fail(BSSE_EINVAL, "radius %g outside 0..1", (double)radius);
    for (int i = 0; i < g->m; ++i)
        if (!std::isfinite(centre[i])) return fail(BSSE_ENOTFINITE, "centre[%d] is not finite", i);
    return BSSE_OK;
}

bsse_status upload_centre(bsse_game *g, const float *centre)
{
    if (!g->centre_dev) HIP_TRY(hipMalloc((void **)&g->centre_dev, (size_t)g->m * sizeof(float)));
    HIP_TRY(hipMemcpyAsync(g->centre_dev, centre, (size_t)g->m * sizeof(float), hipMemcpyHostToDevice, g->stream));
    HIP_TRY(hipStreamSynchronize(g->stream));          // the host array is the caller's again
    return BSSE_OK;
}

bsse_status lattice_impl(bsse_game *g, int N, const float *centre, float radius, int64_t *count_out);

}  // namespace

extern "C" bsse_status bsse_lattice(bsse_game *g, int N, int64_t *count_out)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (!count_out) return fail(BSSE_EINVAL, "count_out is NULL");
    return lattice_impl(g, N, nullptr, 1.0f, count_out);
}

extern "C" bsse_status bsse_lattice_around(bsse_game *g, int N, const float *centre, float radius,
                                           int64_t *count_out)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (!count_out) return fail(BSSE_EINVAL, "count_out is NULL");
    bsse_status st = check_around(g, centre, radius);
    if (st != BSSE_OK) return st;
    return lattice_impl(g, N, centre, radius, count_out);
}

namespace {

bsse_status lattice_impl(bsse_game *g, int N, const float *centre, float radius, int64_t *count_out)
{
    int64_t cnt = 0;
    bsse_status st = bsse_lattice_count(g->m, N, &cnt);
    if (st != BSSE_OK) return st;
    const int m = g->m;
    const size_t tab_elems = (size_t)(m + 1) * (N + 1);
    if (tab_elems > (1ull << 27)) return fail(BSSE_EOVERFLOW, "lattice table of %zu entries is too large", tab_elems);
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");
    if ((st = ensure_gen(g, (unsigned long long)cnt)) != BSSE_OK) return st;
    if (g->lat_table_N != N) {                    // (the table of the last resolution stays on the device)
        // W(R,q) = C(R+q-1, q-1) for q = 0..m, R = 0..N by Pascal's rule; every entry <= cnt
        std::vector<unsigned long long> tab(tab_elems, 0ull);
        for (int q = 1; q <= m; ++q)
            for (int R = 0; R <= N; ++R) {
                unsigned long long v;
                if (q == 1 || R == 0) v = 1;
                else v = tab[(size_t)q * (N + 1) + R - 1] + tab[(size_t)(q - 1) * (N + 1) + R];
                tab[(size_t)q * (N + 1) + R] = v;
            }
        g->lat_table_N = -1;
        if (tab_elems * 8 > g->lat_table_cap) {
            HIP_TRY(hipStreamSynchronize(g->stream));
            (void)hipFree(g->lat_table);
            g->lat_table = nullptr; g->lat_table_cap = 0;
            HIP_TRY(hipMalloc((void **)&g->lat_table, tab_elems * 8));
            g->lat_table_cap = tab_elems * 8;
        }
        HIP_TRY(hipMemcpyAsync(g->lat_table, tab.data(), tab_elems * 8, hipMemcpyHostToDevice, g->stream));
        HIP_TRY(hipStreamSynchronize(g->stream));     // `tab` is pageable and dies with this block
        g->lat_table_N = N;
    }
    if (centre && (st = upload_centre(g, centre)) != BSSE_OK) return st;
    HIP_TRY(launch_lattice(g->lat_table, m, N, cnt, centre ? g->centre_dev : nullptr, radius, g->gen, g->stream));
    g->gen_count = cnt;
    *count_out = cnt;
    return BSSE_OK;
}

bsse_status dirichlet_impl(bsse_game *g, uint64_t seed, int64_t first, int64_t count, const float *centre,
                           float radius, float *out_dev);

}  // namespace

extern "C" bsse_status bsse_dirichlet(bsse_game *g, uint64_t seed, int64_t first, int64_t count,
                                      float *out_dev)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    return dirichlet_impl(g, seed, first, count, nullptr, 1.0f, out_dev);
}

extern "C" bsse_status bsse_dirichlet_around(bsse_game *g, uint64_t seed, int64_t first, int64_t count,
                                             const float *centre, float radius, float *out_dev)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    bsse_status st = check_around(g, centre, radius);
    if (st != BSSE_OK) return st;
    return dirichlet_impl(g, seed, first, count, centre, radius, out_dev);
}

namespace {

bsse_status dirichlet_impl(bsse_game *g, uint64_t seed, int64_t first, int64_t count, const float *centre,
                           float radius, float *out_dev)
{
    if (first < 0 || count < 0) return fail(BSSE_EINVAL, "first and count must be >= 0");
    if (count > CHUNK_MAX) return fail(BSSE_EOVERFLOW, "count exceeds 2^31 rows per call");
    if (first > INT64_MAX - count) return fail(BSSE_EOVERFLOW, "first + count overflows");
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");
    float *dst = out_dev;
    if (!dst) {
        bsse_status st = ensure_gen(g, (unsigned long long)count);
        if (st != BSSE_OK) return st;
        dst = g->gen;
    }
    if (centre) {
        bsse_status st = upload_centre(g, centre);
        if (st != BSSE_OK) return st;
    }
    HIP_TRY(launch_dirichlet(seed, first, count, g->m, centre ? g->centre_dev : nullptr, radius, dst, g->stream));
    if (!out_dev) g->gen_count = count;
    return BSSE_OK;
}

}  // namespace

extern "C" bsse_status bsse_candidates(bsse_game *g, const float **dev_out, int64_t *count_out)
{
    g_err[0] = 0;
    if (!g || !dev_out || !count_out) return fail(BSSE_EINVAL, "NULL argument");
    if (g->gen_count < 0) return fail(BSSE_ESTATE, "no candidate set has been generated on this handle");
    *dev_out = g->gen;
    *count_out = g->gen_count;
    return BSSE_OK;
}

// -------------------------------------------------------------------------------- sweep
extern "C" bsse_status bsse_sweep_reset(bsse_game *g)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");
    g->fresh = true;          // consumed by the merge kernel of the next chunk: no launch here
    g->result_valid = false;
    g->n_evals = 0;
    return BSSE_OK;
}

static bsse_status resolve_candidates(bsse_game *g, const float **X, int64_t *count)
{
    if (*count < 0) return fail(BSSE_EINVAL, "count must be >= 0");
    if (!*X) {
        if (g->gen_count < 0)
            return fail(BSSE_ESTATE, "candidates is NULL but no set has been generated on this handle");
        if (*count != 0 && *count != g->gen_count)
            return fail(BSSE_EINVAL, "count %lld does not match the generated set (%lld)",
                        (long long)*count, g->gen_count);
        *X = g->gen;
        *count = g->gen_count;
    }
    if (*count > CHUNK_MAX) return fail(BSSE_EOVERFLOW, "count exceeds 2^31 rows per call");
    const uintptr_t need = (g->m % 4 == 0) ? 15 : 3;      // whole rows of 16 bytes keep 16-byte alignment
    if (((uintptr_t)*X & need) != 0)
        return fail(BSSE_EINVAL, "candidates must be %d-byte aligned", (int)need + 1);
    return BSSE_OK;
}

namespace {

// One chunk through the sweep kernel and the merge into the running best.  a.X / a.gen*, a.count
// and a.index_base are set by the caller; the device is current.
bool on_small_kernel(const bsse_game *g)
{
    return g->path != PATH_VALU && mfma_is_small(g->view.variant);
}

// The caller's stream waits for whatever the handle's own streams still have in flight.
bsse_status join_aux(bsse_game *g)
{
    for (int q = 0; q < 2; ++q) {
        if (!g->aux_used[q]) continue;
        HIP_TRY(hipEventRecord(g->aux_join[q], g->aux[q]));
        HIP_TRY(hipStreamWaitEvent(g->stream, g->aux_join[q], 0));
        g->aux_used[q] = false;
    }
    return BSSE_OK;
}

bsse_status ensure_aux(bsse_game *g)
{
    if (g->aux[0]) return BSSE_OK;
    HIP_TRY(hipEventCreateWithFlags(&g->aux_fork, hipEventDisableTiming));
    for (int q = 0; q < 2; ++q) {
        HIP_TRY(hipStreamCreateWithFlags(&g->aux[q], hipStreamNonBlocking));     // default priority
        HIP_TRY(hipEventCreateWithFlags(&g->aux_join[q], hipEventDisableTiming));
    }
    return BSSE_OK;
}

bsse_status sweep_chunk_impl(bsse_game *g, SweepArgs a)
{
    bsse_status st;
    const long long count = a.count;
    const bool small = on_small_kernel(g);
    long long nblocks = 0;
    hipStream_t stream = g->stream;
    if (small) {
        // every workgroup keeps its own running best over the chunks: nothing but the sweep
        // kernel runs per chunk; bsse_sweep_result folds
        if (g->fresh) {
            if ((st = join_aux(g)) != BSSE_OK) return st;        // an abandoned sweep may still be running
            g->epoch += 1;
            if (g->epoch == 0) g->epoch = 1;         // 0 is the mark of a slot never written
            g->fold_first = true;
            g->chunk_seq = 0;
            if (g->ties_dirty) HIP_TRY(launch_clear_u64(g->w.tie_counter, g->stream));   // an abandoned sweep's
        }
        int set = g->w.slot_sets - 1;                // the caller's stream (the last set)
        if (a.gen && g->chunk_seq > 0 && g->w.slot_sets == 3) {
            // (the first chunk stays on the caller's stream, so a one-chunk sweep pays for no events)
            if ((st = ensure_aux(g)) != BSSE_OK) return st;
            set = (int)(g->chunk_seq & 1u);
            if (!g->aux_used[set]) {
                HIP_TRY(hipEventRecord(g->aux_fork, g->stream));
                HIP_TRY(hipStreamWaitEvent(g->aux[set], g->aux_fork, 0));
                g->aux_used[set] = true;
            }
            stream = g->aux[set];
        }
        g->chunk_seq += 1;
        a.small.slots = g->w.slots + (size_t)set * small_num_slots(); a.small.epoch = g->epoch;
        a.tie_counter = g->w.tie_counter;
    } else {
        nblocks = sweep_blocks(g, count);
        if ((st = ensure_blocks(g, nblocks)) != BSSE_OK) return st;
        a.blk_v = g->w.blk_v; a.blk_i = g->w.blk_i; a.tie_counter = g->w.tie_counter;
    }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (g->timing) {
        if ((st = take_event(g, &e0)) != BSSE_OK) return st;
        if ((st = take_event(g, &e1)) != BSSE_OK) { g->ev_pool.push_back(e0); return st; }
        HIP_TRY(hipEventRecord(e0, stream));
    }
    hipError_t le = launch_sweep_on(g, a, false, stream);
    if (g->timing) {
        (void)hipEventRecord(e1, stream);
        g->ev.push_back(e0); g->ev.push_back(e1);
    }
    HIP_TRY(le);
    if (small) {
        g->fold_pending = true; g->ties_dirty = true;
    } else {
        HIP_TRY(launch_reduce_merge(g->w.blk_v, g->w.blk_i, nblocks, a.X, a.index_base, g->m,
                                    g->fresh ? 1 : 0, g->w.tie_counter, g->w.run, &g->h_out->run, g->w.best_x,
                                    g->stream));
    }
    g->fresh = false;
    g->result_valid = false;  // until bsse_sweep_result has brought the new state to the host
    g->n_evals += count * g->K;
    return BSSE_OK;
}

// Small-game kernel: fold the workgroups' running bests into the handle's result (value, index,
// row, best responses, tie count).  No-op when nothing was swept since the last fold.
bsse_status fold_small(bsse_game *g)
{
    if (!on_small_kernel(g) || !g->fold_pending) return BSSE_OK;
    bsse_status st = join_aux(g);
    if (st != BSSE_OK) return st;
    FinishArgs f{};
    f.slots = g->w.slots; f.nslots = g->w.slot_sets * small_num_slots(); f.epoch = g->epoch;
    f.first = g->fold_first ? 1 : 0;
    f.tie_counter = g->w.tie_counter;
    f.run = g->w.run; f.run_host = &g->h_out->run; f.best_x = g->w.best_x;
    f.win_v = &g->h_out->fin_v; f.win_br = g->h_br;
    HIP_TRY(launch_finish_small(g->view, f, g->stream));
    g->fold_pending = false; g->fold_first = false; g->ties_dirty = false;
    return BSSE_OK;
}

bool fuses_generation(const bsse_game *g) { return on_small_kernel(g); }

bsse_status check_rows(int64_t first, int64_t count)
{
    if (first < 0 || count < 0) return fail(BSSE_EINVAL, "first and count must be >= 0");
    if (count > CHUNK_MAX) return fail(BSSE_EOVERFLOW, "count exceeds 2^31 rows per call");
    if (first > INT64_MAX - count) return fail(BSSE_EOVERFLOW, "first + count overflows");
    return BSSE_OK;
}

}  // namespace

extern "C" bsse_status bsse_sweep_chunk(bsse_game *g, const float *candidates_dev, int64_t count,
                                        int64_t index_base)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (index_base < 0) return fail(BSSE_EINVAL, "index_base must be >= 0");
    bsse_status st = resolve_candidates(g, &candidates_dev, &count);
    if (st != BSSE_OK) return st;
    if (index_base > INT64_MAX - count) return fail(BSSE_EOVERFLOW, "index_base + count overflows");
    if (count == 0) return BSSE_OK;
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");
    SweepArgs a{};
    a.X = candidates_dev; a.count = count; a.index_base = index_base;
    return sweep_chunk_impl(g, a);
}

extern "C" bsse_status bsse_sweep_dirichlet_chunk(bsse_game *g, uint64_t seed, int64_t first,
                                                  int64_t count, int64_t index_base)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (index_base < 0) return fail(BSSE_EINVAL, "index_base must be >= 0");
    bsse_status st = check_rows(first, count);
    if (st != BSSE_OK) return st;
    if (index_base > INT64_MAX - count) return fail(BSSE_EOVERFLOW, "index_base + count overflows");
    if (count == 0) return BSSE_OK;
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");
    if (fuses_generation(g)) {
        SweepArgs a{};
        a.count = count; a.index_base = index_base;
        a.gen = 1; a.gen_k0 = (unsigned)(seed & 0xFFFFFFFFull); a.gen_k1 = (unsigned)(seed >> 32);
        a.gen_first = first;
        return sweep_chunk_impl(g, a);
    }
    // other shapes: the rows pass through a staging buffer of the handle (at most 2^26 floats),
    // piece by piece on the handle's stream
    long long piece = (1LL << 26) / g->m;
    if (piece > count) piece = count;
    const size_t bytes = (size_t)piece * g->m * sizeof(float);
    if (bytes > g->stage_cap) {
        HIP_TRY(hipStreamSynchronize(g->stream));
        (void)hipFree(g->stage);
        g->stage = nullptr; g->stage_cap = 0;
        HIP_TRY(hipMalloc((void **)&g->stage, bytes));
        g->stage_cap = bytes;
    }
    for (long long base = 0; base < count; base += piece) {
        const long long rows = count - base < piece ? count - base : piece;
        HIP_TRY(launch_dirichlet(seed, first + base, rows, g->m, nullptr, 1.0f, g->stage, g->stream));
        SweepArgs a{};
        a.X = g->stage; a.count = rows; a.index_base = index_base + base;
        if ((st = sweep_chunk_impl(g, a)) != BSSE_OK) return st;
    }
    return BSSE_OK;
}

extern "C" bsse_status bsse_sweep_dirichlet(bsse_game *g, uint64_t seed, int64_t first, int64_t count,
                                            bsse_result *res, int32_t *best_response_out)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (!res) return fail(BSSE_EINVAL, "res is NULL");
    bsse_status st = check_rows(first, count);
    if (st != BSSE_OK) return st;
    if ((st = bsse_sweep_reset(g)) != BSSE_OK) return st;
    if ((st = bsse_sweep_dirichlet_chunk(g, seed, first, count, 0)) != BSSE_OK) return st;
    return bsse_sweep_result(g, res, best_response_out);
}

extern "C" bsse_status bsse_sweep_result(bsse_game *g, bsse_result *res, int32_t *best_response_out)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (!res) return fail(BSSE_EINVAL, "res is NULL");
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");
    if (g->fresh) {                        // nothing swept since the last reset
        HIP_TRY(hipStreamSynchronize(g->stream));
        res->best_value = 0.0; res->best_index = -1; res->n_evals = 0; res->n_tie_evals = 0;
        return BSSE_OK;
    }
    // best responses of the winner: the same kernel, one row, per-candidate outputs written
    // straight into pinned host memory (the small-game kernel carries them with its records)
    if (on_small_kernel(g)) {
        bsse_status st = fold_small(g);
        if (st != BSSE_OK) return st;
    } else {
        SweepArgs a{};
        a.X = g->w.best_x; a.count = 1; a.index_base = 0;
        a.V_out = &g->h_out->fin_v; a.br_out = g->h_br;
        // one row against every type: the general matrix-core kernel spreads the types over the chip
        if (g->path != PATH_VALU && mfma_slices_types(g->view.variant)) a.l_out = g->w.win_l;
        HIP_TRY(launch_sweep(g, a, true));
    }
    HIP_TRY(hipStreamSynchronize(g->stream));
    const bool has = g->h_out->run.has != 0;
    if (has && !(g->h_out->fin_v == g->h_out->run.value))
        return fail(BSSE_EDEVICE, "internal: re-evaluated winner value %.9g differs from swept value %.9g",
                    (double)g->h_out->fin_v, (double)g->h_out->run.value);
    res->best_value = has ? (double)g->h_out->run.value : 0.0;
    res->best_index = has ? (int64_t)g->h_out->run.index : -1;
    res->n_evals = g->n_evals;
    res->n_tie_evals = (int64_t)g->h_out->run.ties;
    if (has && best_response_out) memcpy(best_response_out, g->h_br, (size_t)g->K * 4);
    g->result_valid = has && !g->w.fixed;
    return BSSE_OK;
}

extern "C" bsse_status bsse_sweep_best_row(bsse_game *g, float *x_out)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (!x_out) return fail(BSSE_EINVAL, "x_out is NULL");
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");
    if (!g->fresh) {
        bsse_status st = fold_small(g);
        if (st != BSSE_OK) return st;
    }
    HIP_TRY(hipStreamSynchronize(g->stream));
    if (g->fresh || !g->h_out->run.has) return fail(BSSE_ESTATE, "no candidate has been swept since the last reset");
    HIP_TRY(hipMemcpy(x_out, g->w.best_x, (size_t)g->m * sizeof(float), hipMemcpyDeviceToHost));
    return BSSE_OK;
}

extern "C" bsse_status bsse_sweep(bsse_game *g, const float *candidates_dev, int64_t count,
                                  bsse_result *res, int32_t *best_response_out)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (!res) return fail(BSSE_EINVAL, "res is NULL");
    {   // argument errors first, before anything is enqueued
        const float *x = candidates_dev;
        int64_t c = count;
        bsse_status st = resolve_candidates(g, &x, &c);
        if (st != BSSE_OK) return st;
    }
    bsse_status st = bsse_sweep_reset(g);
    if (st != BSSE_OK) return st;
    if ((st = bsse_sweep_chunk(g, candidates_dev, count, 0)) != BSSE_OK) return st;
    return bsse_sweep_result(g, res, best_response_out);
}

// bsse_sweep with every piece of device scratch taken from the static array: no allocation of any
// kind happens in this call (device, pinned host or stream/event objects).
extern "C" bsse_status bsse_sweep_static(bsse_game *g, const float *candidates_dev, int64_t count,
                                         bsse_result *res, int32_t *best_response_out)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (!res) return fail(BSSE_EINVAL, "res is NULL");
    if (!candidates_dev) return fail(BSSE_EINVAL, "candidates is NULL (the static sweep takes an explicit buffer)");
    {
        const float *x = candidates_dev;
        int64_t c = count;
        bsse_status st = resolve_candidates(g, &x, &c);
        if (st != BSSE_OK) return st;
    }
    const bool small = on_small_kernel(g);
    if (!small && sweep_blocks(g, count) > STATIC_MAX_BLOCKS)
        return fail(BSSE_EOVERFLOW, "%lld candidates need %lld workgroup records; the static scratch holds %lld "
                    "(sweep in pieces, or use bsse_sweep)", (long long)count, sweep_blocks(g, count),
                    STATIC_MAX_BLOCKS);
    if (small && small_num_slots() > STATIC_MAX_SLOTS)
        return fail(BSSE_EOVERFLOW, "the static scratch holds %d running-best slots, %d needed", STATIC_MAX_SLOTS,
                    small_num_slots());
    if (g->m > STATIC_MAX_M || g->K > STATIC_MAX_K)
        return fail(BSSE_EOVERFLOW, "the static scratch holds rows of %d and %d types", STATIC_MAX_M, STATIC_MAX_K);
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");
    unsigned char *ptr = nullptr;
    bsse_status st = static_scratch(g->device, &ptr);
    if (st != BSSE_OK) return st;

    // the handle works on the static scratch for the length of this call; its own sweep state
    // is what bsse_sweep leaves behind as well: reset
    struct Swap {
        bsse_game *g; Work own; bool timing, ties_dirty;
        ~Swap()
        {
            g->w = own; g->timing = timing; g->ties_dirty = ties_dirty;
            g->fresh = true; g->fold_pending = false; g->result_valid = false; g->n_evals = 0;
        }
    } swap{ g, g->w, g->timing, g->ties_dirty };
    Work w;
    w.run = reinterpret_cast<RunningBest *>(ptr + ST_OFF_RUN);
    w.tie_counter = reinterpret_cast<unsigned long long *>(ptr + ST_OFF_TIES);
    w.best_x = reinterpret_cast<float *>(ptr + ST_OFF_BESTX);
    w.win_l = reinterpret_cast<float *>(ptr + ST_OFF_WINL);
    w.blk_v = reinterpret_cast<float *>(ptr + ST_OFF_BLKV);
    w.blk_i = reinterpret_cast<long long *>(ptr + ST_OFF_BLKI);
    w.blk_cap = STATIC_MAX_BLOCKS;
    w.slots = small ? reinterpret_cast<SmallSlot *>(ptr + ST_OFF_SLOTS) : nullptr;
    w.slot_sets = small ? 1 : 0;
    w.fixed = true;
    g->w = w;
    g->timing = false;              // (event pairs would be created on demand)
    g->ties_dirty = false;
    // the array keeps the last call's contents, possibly another handle's: the running best, the
    // tie counter and (small-game kernel) the slots' epochs start from zero.  A fill kernel, not a
    // memset node, so that the call stays safe to capture.
    HIP_TRY(launch_fill_zero(ptr, ST_OFF_BESTX, g->stream));
    if (small) HIP_TRY(launch_fill_zero(ptr + ST_OFF_SLOTS, (size_t)small_num_slots() * sizeof(SmallSlot), g->stream));
    if ((st = bsse_sweep_reset(g)) != BSSE_OK) return st;
    if ((st = bsse_sweep_chunk(g, candidates_dev, count, 0)) != BSSE_OK) return st;
    return bsse_sweep_result(g, res, best_response_out);
}

extern "C" bsse_status bsse_eval(bsse_game *g, const float *candidates_dev, int64_t count,
                                 float *values_dev_out, int32_t *br_dev_out)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    bsse_status st = resolve_candidates(g, &candidates_dev, &count);
    if (st != BSSE_OK) return st;
    if (count == 0 || (!values_dev_out && !br_dev_out)) return BSSE_OK;
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");
    SweepArgs a{};
    a.X = candidates_dev; a.count = count; a.index_base = 0;
    a.V_out = values_dev_out; a.br_out = br_dev_out;
    HIP_TRY(launch_sweep(g, a, true));
    return BSSE_OK;
}

// ------------------------------------------------------------------------ prior batch
extern "C" bsse_status bsse_sweep_priors(bsse_game *g, const float *candidates_dev, int64_t count,
                                         const float *priors, int P, bsse_result *res,
                                         int32_t *best_response_out)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (!priors) return fail(BSSE_EINVAL, "priors is NULL");
    if (!res) return fail(BSSE_EINVAL, "res is NULL");
    if (P < 1 || P > 65536) return fail(BSSE_EINVAL, "P = %d outside 1..65536", P);
    const int K = g->K, m = g->m;
    for (int p = 0; p < P; ++p) {
        double psum = 0.0;
        for (int t = 0; t < K; ++t) {
            const float v = priors[(size_t)p * K + t];
            if (!std::isfinite(v)) return fail(BSSE_ENOTFINITE, "priors[%d][%d] is not finite", p, t);
            if (v < 0.0f) return fail(BSSE_EINVAL, "priors[%d][%d] is negative", p, t);
            psum += (double)v;
        }
        if (std::fabs(psum - 1.0) > 1e-6)
            return fail(BSSE_EINVAL, "priors[%d] sums to %.9g, not 1", p, psum);
    }
    bsse_status st = resolve_candidates(g, &candidates_dev, &count);
    if (st != BSSE_OK) return st;
    if (count == 0) {
        for (int p = 0; p < P; ++p) { res[p].best_value = 0.0; res[p].best_index = -1; res[p].n_evals = 0; res[p].n_tie_evals = 0; }
        return BSSE_OK;
    }
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");

    // the leader-payoff matrix is built chunk by chunk: at most 2^28 entries (1 GiB) at a time
    long long chunk = (1LL << 28) / K;
    if (chunk < 4096) chunk = 4096;
    if (chunk > count) chunk = count;
    const int nblocks = prior_batch_blocks(chunk, P);
    PriorScratch &w = g->pri;
    auto grow = [&](void **ptr, size_t *cap, size_t bytes) -> bsse_status {
        if (bytes <= *cap) return BSSE_OK;
        HIP_TRY(hipStreamSynchronize(g->stream));      // nothing enqueued may still use the old block
        (void)hipFree(*ptr);
        *ptr = nullptr; *cap = 0;
        HIP_TRY(hipMalloc(ptr, bytes));
        *cap = bytes;
        return BSSE_OK;
    };
    if ((st = grow((void **)&w.L, &w.cap_L, (size_t)chunk * K * sizeof(float))) != BSSE_OK) return st;
    if ((st = grow((void **)&w.priors, &w.cap_priors, (size_t)P * K * sizeof(float))) != BSSE_OK) return st;
    if ((st = grow((void **)&w.blk_v, &w.cap_blk_v, (size_t)nblocks * P * sizeof(float))) != BSSE_OK) return st;
    if ((st = grow((void **)&w.blk_i, &w.cap_blk_i, (size_t)nblocks * P * sizeof(long long))) != BSSE_OK) return st;
    if ((st = grow((void **)&w.run, &w.cap_run, (size_t)P * sizeof(PriorBest))) != BSSE_OK) return st;
    if ((st = grow((void **)&w.rows, &w.cap_rows, (size_t)P * m * sizeof(float))) != BSSE_OK) return st;
    if ((st = grow((void **)&w.br, &w.cap_br, (size_t)P * K * sizeof(int32_t))) != BSSE_OK) return st;
    if ((st = grow((void **)&w.ties, &w.cap_ties, sizeof(unsigned long long))) != BSSE_OK) return st;
    // pinned staging, so that the copies below are asynchronous and the call waits once, at the end
    const size_t in_bytes = (size_t)P * K * sizeof(float);
    const size_t off_run = 0, off_br = (size_t)P * sizeof(PriorBest), off_ties = off_br + (size_t)P * K * sizeof(int32_t);
    const size_t out_bytes = off_ties + sizeof(unsigned long long);
    const size_t host_bytes = in_bytes > out_bytes ? in_bytes : out_bytes;
    if (host_bytes > w.cap_host) {
        HIP_TRY(hipStreamSynchronize(g->stream));
        if (w.host) (void)hipHostFree(w.host);
        w.host = nullptr; w.cap_host = 0;
        if (hipHostMalloc((void **)&w.host, host_bytes, hipHostMallocDefault) != hipSuccess)
            return fail(BSSE_ENOMEM, "hipHostMalloc of %zu bytes failed", host_bytes);
        w.cap_host = host_bytes;
    }
    memcpy(w.host, priors, in_bytes);
    HIP_TRY(hipMemcpyAsync(w.priors, w.host, in_bytes, hipMemcpyHostToDevice, g->stream));
    HIP_TRY(launch_clear_u64(w.ties, g->stream));                // a counter of its own
    for (long long base = 0; base < count; base += chunk) {
        const long long rows = count - base < chunk ? count - base : chunk;
        SweepArgs a{};
        a.X = candidates_dev + base * m; a.count = rows; a.index_base = base;
        a.l_out = w.L; a.tie_counter = w.ties;
        HIP_TRY(launch_sweep(g, a, true));
        HIP_TRY(launch_prior_batch(w.L, rows, base, K, w.priors, P, base == 0 ? 1 : 0, w.blk_v, w.blk_i,
                                   w.run, g->stream));
    }
    // best responses of the P winners: their rows, evaluated once more with per-candidate outputs
    HIP_TRY(launch_gather_rows(candidates_dev, w.run, P, m, w.rows, g->stream));
    {
        SweepArgs a{};
        a.X = w.rows; a.count = P; a.index_base = 0; a.br_out = w.br;
        HIP_TRY(launch_sweep(g, a, true));
    }
    // (the staging buffer is free again once the copy of the priors has run: same stream)
    HIP_TRY(hipMemcpyAsync(w.host + off_run, w.run, (size_t)P * sizeof(PriorBest), hipMemcpyDeviceToHost, g->stream));
    HIP_TRY(hipMemcpyAsync(w.host + off_br, w.br, (size_t)P * K * sizeof(int32_t), hipMemcpyDeviceToHost, g->stream));
    HIP_TRY(hipMemcpyAsync(w.host + off_ties, w.ties, sizeof(unsigned long long), hipMemcpyDeviceToHost, g->stream));
    HIP_TRY(hipStreamSynchronize(g->stream));
    const PriorBest *run = reinterpret_cast<const PriorBest *>(w.host + off_run);
    unsigned long long ties = 0;
    memcpy(&ties, w.host + off_ties, sizeof(ties));
    for (int p = 0; p < P; ++p) {
        res[p].best_value = run[p].has ? (double)run[p].value : 0.0;
        res[p].best_index = run[p].has ? (int64_t)run[p].index : -1;
        res[p].n_evals = (int64_t)count * K;
        res[p].n_tie_evals = (int64_t)ties;
    }
    if (best_response_out) memcpy(best_response_out, w.host + off_br, (size_t)P * K * sizeof(int32_t));
    return BSSE_OK;
}

// --------------------------------------------------------------------------------- top-k
namespace {

struct DevView {                     // a block of handle-owned scratch
    void *p = nullptr;
    template <typename T> T *as() const { return reinterpret_cast<T *>(p); }
};

struct DevBuf {                      // device scratch of one call, released on every exit path
    void *p = nullptr;
    ~DevBuf() { (void)hipFree(p); }
    template <typename T> T *as() const { return reinterpret_cast<T *>(p); }
};

}  // namespace

extern "C" bsse_status bsse_sweep_topk(bsse_game *g, const float *candidates_dev, int64_t count, int k,
                                       double *values_out, int64_t *indices_out,
                                       int32_t *best_response_out, int *found_out)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (!values_out || !indices_out || !found_out) return fail(BSSE_EINVAL, "NULL argument");
    if (k < 1 || k > 256) return fail(BSSE_EINVAL, "k = %d outside 1..256", k);
    bsse_status st = resolve_candidates(g, &candidates_dev, &count);
    if (st != BSSE_OK) return st;
    if (count == 0) { *found_out = 0; return BSSE_OK; }
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");
    const int m = g->m, K = g->K;

    const long long chunk = count < (1LL << 26) ? count : (1LL << 26);
    const long long nchunks = (count + chunk - 1) / chunk;
    const long long rec0 = topk_level_blocks(chunk) * k;          // records after the first level
    // scratch of the handle, grown on demand (allocating and freeing per call costs more than the call)
    DevView V, av, ai, bv, bi, wv, wi, rows, br;
    {
        DevView *views[9] = { &V, &av, &ai, &bv, &bi, &wv, &wi, &rows, &br };
        const size_t need[9] = { (size_t)chunk * sizeof(float), (size_t)rec0 * sizeof(float),
                                 (size_t)rec0 * sizeof(long long), (size_t)rec0 * sizeof(float),
                                 (size_t)rec0 * sizeof(long long), (size_t)(nchunks + 1) * k * sizeof(float),
                                 (size_t)(nchunks + 1) * k * sizeof(long long), (size_t)k * m * sizeof(float),
                                 (size_t)k * K * sizeof(int32_t) };
        for (int q = 0; q < 9; ++q) {
            if (need[q] > g->topk.cap[q]) {
                HIP_TRY(hipStreamSynchronize(g->stream));   // nothing enqueued may still use the old block
                (void)hipFree(g->topk.p[q]);
                g->topk.p[q] = nullptr; g->topk.cap[q] = 0;
                HIP_TRY(hipMalloc(&g->topk.p[q], need[q]));
                g->topk.cap[q] = need[q];
            }
            views[q]->p = g->topk.p[q];
        }
    }

    // levels from `n` (value, index) records in (sv, si) down to k records, written to (dv, di)
    auto reduce_to = [&](const float *sv, const long long *si, long long n, long long index_base,
                         float *dv, long long *di) -> bsse_status {
        float *pv[2] = { av.as<float>(), bv.as<float>() };
        long long *pi[2] = { ai.as<long long>(), bi.as<long long>() };
        int cur = 0;
        for (;;) {
            const long long nb = topk_level_blocks(n);
            float *ov = nb == 1 ? dv : pv[cur];
            long long *oi = nb == 1 ? di : pi[cur];
            HIP_TRY(launch_topk_level(sv, si, n, index_base, k, ov, oi, g->stream));
            if (nb == 1) return BSSE_OK;
            sv = ov; si = oi; n = nb * k; cur ^= 1;
        }
    };
    for (long long c = 0; c < nchunks; ++c) {
        const long long base = c * chunk, n = count - base < chunk ? count - base : chunk;
        SweepArgs a{};
        a.X = candidates_dev + base * m; a.count = n; a.index_base = 0; a.V_out = V.as<float>();
        HIP_TRY(launch_sweep(g, a, true));
        if ((st = reduce_to(V.as<float>(), nullptr, n, base, wv.as<float>() + c * k,
                            wi.as<long long>() + c * k)) != BSSE_OK) return st;
    }
    float *fv = wv.as<float>();
    long long *fi = wi.as<long long>();
    if (nchunks > 1) {
        fv += nchunks * k; fi += nchunks * k;
        if ((st = reduce_to(wv.as<float>(), wi.as<long long>(), nchunks * k, 0, fv, fi)) != BSSE_OK) return st;
    }
    // best responses of the survivors: their rows, evaluated once more with per-candidate outputs
    HIP_TRY(launch_gather_indexed_rows(candidates_dev, fi, k, m, rows.as<float>(), g->stream));
    {
        SweepArgs a{};
        a.X = rows.as<float>(); a.count = k; a.index_base = 0; a.br_out = br.as<int32_t>();
        HIP_TRY(launch_sweep(g, a, true));
    }
    std::vector<float> hv((size_t)k);
    std::vector<long long> hi((size_t)k);
    std::vector<int32_t> hb(best_response_out ? (size_t)k * K : 0);
    HIP_TRY(hipMemcpyAsync(hv.data(), fv, (size_t)k * sizeof(float), hipMemcpyDeviceToHost, g->stream));
    HIP_TRY(hipMemcpyAsync(hi.data(), fi, (size_t)k * sizeof(long long), hipMemcpyDeviceToHost, g->stream));
    if (best_response_out)
        HIP_TRY(hipMemcpyAsync(hb.data(), br.p, hb.size() * sizeof(int32_t), hipMemcpyDeviceToHost, g->stream));
    HIP_TRY(hipStreamSynchronize(g->stream));
    int found = 0;
    while (found < k && hi[found] != LLONG_MAX) ++found;
    for (int r = 0; r < found; ++r) { values_out[r] = (double)hv[r]; indices_out[r] = (int64_t)hi[r]; }
    if (best_response_out) memcpy(best_response_out, hb.data(), (size_t)found * K * sizeof(int32_t));
    *found_out = found;
    return BSSE_OK;
}

// ------------------------------------------------------------------------------- refinement
extern "C" bsse_status bsse_refine(bsse_game *g, int k, int rounds, int lattice_N, int64_t cloud_count,
                                   uint64_t seed, float radius, float shrink, float *x_out,
                                   bsse_result *res, int32_t *best_response_out)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (!x_out || !res) return fail(BSSE_EINVAL, "NULL argument");
    if (k < 1 || k > 256) return fail(BSSE_EINVAL, "k = %d outside 1..256", k);
    if (rounds < 1 || rounds > 64) return fail(BSSE_EINVAL, "rounds = %d outside 1..64", rounds);
    if ((lattice_N > 0) == (cloud_count > 0))
        return fail(BSSE_EINVAL, "give either lattice_N > 0 or cloud_count > 0");
    if (!(radius > 0.0f && radius <= 1.0f) || !(shrink > 0.0f && shrink <= 1.0f))
        return fail(BSSE_EINVAL, "radius and shrink must lie in (0, 1]");
    if (g->gen_count <= 0) return fail(BSSE_ESTATE, "no candidate set has been generated on this handle");
    const int m = g->m, K = g->K;
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");

    // survivors: value, row, best responses; kept sorted by (value desc, order of discovery)
    struct Survivor { double v; std::vector<float> x; std::vector<int32_t> br; };
    std::vector<Survivor> pool;
    std::vector<double> vals((size_t)k);
    std::vector<int64_t> idx((size_t)k);
    std::vector<int32_t> brs((size_t)k * K);
    long long evals = 0;
    // the k best of the handle's current set, with their rows, into `into`
    auto harvest = [&](std::vector<Survivor> &into) -> bsse_status {
        int found = 0;
        bsse_status st = bsse_sweep_topk(g, nullptr, 0, k, vals.data(), idx.data(), brs.data(), &found);
        if (st != BSSE_OK) return st;
        evals += (long long)g->gen_count * K;
        for (int r = 0; r < found; ++r) {
            Survivor sv;
            sv.v = vals[r];
            sv.x.resize((size_t)m);
            sv.br.assign(brs.begin() + (size_t)r * K, brs.begin() + (size_t)(r + 1) * K);
            HIP_TRY(hipMemcpy(sv.x.data(), g->gen + (size_t)idx[r] * m, (size_t)m * sizeof(float),
                              hipMemcpyDeviceToHost));
            into.push_back(std::move(sv));
        }
        return BSSE_OK;
    };
    auto keep_best = [&](std::vector<Survivor> &v) {
        std::stable_sort(v.begin(), v.end(), [](const Survivor &a, const Survivor &b) { return a.v > b.v; });
        // the same point may be found from two centres: keep one
        std::vector<Survivor> out;
        for (auto &sv : v) {
            bool dupl = false;
            for (auto &o : out) if (o.x == sv.x) { dupl = true; break; }
            if (!dupl) out.push_back(std::move(sv));
            if ((int)out.size() == k) break;
        }
        v.swap(out);
    };
    bsse_status st;
    try {
        if ((st = harvest(pool)) != BSSE_OK) return st;
        keep_best(pool);
        float rad = radius;
        for (int round = 0; round < rounds; ++round) {
            std::vector<Survivor> next = pool;             // a centre survives unless it is beaten
            for (size_t c = 0; c < pool.size(); ++c) {
                if (lattice_N > 0) {
                    int64_t cnt = 0;
                    st = bsse_lattice_around(g, lattice_N, pool[c].x.data(), rad, &cnt);
                } else {
                    st = bsse_dirichlet_around(g, seed + (uint64_t)round * 1000003ull + c, 0, cloud_count,
                                               pool[c].x.data(), rad, nullptr);
                }
                if (st != BSSE_OK) return st;
                if ((st = harvest(next)) != BSSE_OK) return st;
            }
            keep_best(next);
            pool.swap(next);
            rad *= shrink;
        }
    } catch (...) { return fail(BSSE_ENOMEM, "host allocation failed"); }
    if (pool.empty()) return fail(BSSE_ESTATE, "the candidate set is empty");
    memcpy(x_out, pool[0].x.data(), (size_t)m * sizeof(float));
    res->best_value = pool[0].v;
    res->best_index = -1;                                  // the point is not a member of one indexed set
    res->n_evals = evals;
    res->n_tie_evals = 0;
    if (best_response_out) memcpy(best_response_out, pool[0].br.data(), (size_t)K * sizeof(int32_t));
    return BSSE_OK;
}

// ----------------------------------------------------------------------------- LP polish
namespace {

bsse_status check_profile(int n, int K, const int32_t *profile)
{
    for (int t = 0; t < K; ++t)
        if (profile[t] < 0 || profile[t] >= n)
            return fail(BSSE_EINVAL, "profile[%d] = %d outside 0..%d", t, (int)profile[t], n - 1);
    return BSSE_OK;
}

constexpr int kPolishRows = 8;       // segment points evaluated by bsse_polish

}  // namespace

extern "C" bsse_status bsse_profile_lp(int m, int n, int K, const float *A, const float *B,
                                       const float *prior, const int32_t *profile, double *x_out,
                                       double *value_out, int *feasible_out)
{
    g_err[0] = 0;
    if (m < 1 || n < 1 || K < 1 || m > 4096 || n > 65535 || K > 65535)
        return fail(BSSE_EINVAL, "bad dimensions m=%d n=%d K=%d", m, n, K);
    if (!A || !B || !prior || !profile || !x_out || !value_out || !feasible_out)
        return fail(BSSE_EINVAL, "NULL argument");
    // the dual tableau holds m rows of 2 + K(n-1) + m columns
    const double cells = (double)m * (2.0 + (double)K * (n - 1) + m);
    if (cells > (double)(1u << 28)) return fail(BSSE_EOVERFLOW, "the program's tableau (%.3g cells) is too large", cells);
    bsse_status st = check_profile(n, K, profile);
    if (st != BSSE_OK) return st;
    const size_t elems = (size_t)K * m * n;
    for (size_t e = 0; e < elems; ++e)
        if (!std::isfinite(A[e]) || !std::isfinite(B[e]))
            return fail(BSSE_ENOTFINITE, "payoff entry %zu is not finite", e);
    for (int t = 0; t < K; ++t)
        if (!std::isfinite(prior[t]) || prior[t] < 0.0f)
            return fail(std::isfinite(prior[t]) ? BSSE_EINVAL : BSSE_ENOTFINITE, "bad prior[%d]", t);
    std::vector<double> x;
    try { x.resize((size_t)m); } catch (...) { return fail(BSSE_ENOMEM, "host allocation failed"); }
    double v = 0.0;
    int rc;
    try { rc = solve_profile_lp(m, n, K, A, B, prior, profile, x.data(), &v); }
    catch (...) { return fail(BSSE_ENOMEM, "host allocation failed"); }
    if (rc == 2) return fail(BSSE_ESTATE, "the simplex method did not converge");
    if (rc == 0) { memcpy(x_out, x.data(), (size_t)m * sizeof(double)); *value_out = v; }
    *feasible_out = rc == 0 ? 1 : 0;
    return BSSE_OK;
}

extern "C" bsse_status bsse_polish(bsse_game *g, const int32_t *profile, float *x_out,
                                   bsse_result *res, int32_t *best_response_out,
                                   double *lp_value_out)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (!x_out || !res) return fail(BSSE_EINVAL, "NULL argument");
    if (!g->result_valid)
        return fail(BSSE_ESTATE, "no sweep result to polish: call bsse_sweep (or _chunk and then _result) first");
    const int m = g->m, n = g->n, K = g->K;
    if (profile) {
        bsse_status st = check_profile(n, K, profile);
        if (st != BSSE_OK) return st;
    }
    const double cells = (double)m * (2.0 + (double)K * (n - 1) + m);
    if (cells > (double)(1u << 28)) return fail(BSSE_EOVERFLOW, "the program's tableau (%.3g cells) is too large", cells);
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");
    HIP_TRY(hipStreamSynchronize(g->stream));            // the winner's row and profile are final
    std::vector<int32_t> prof((size_t)K);
    std::vector<float> start((size_t)m), rows((size_t)kPolishRows * m), vals((size_t)kPolishRows);
    std::vector<int32_t> brs((size_t)kPolishRows * K);
    std::vector<double> x((size_t)m);
    memcpy(prof.data(), profile ? profile : g->h_br, (size_t)K * sizeof(int32_t));
    HIP_TRY(hipMemcpy(start.data(), g->w.best_x, (size_t)m * sizeof(float), hipMemcpyDeviceToHost));
    double v_lp = 0.0;
    const int rc = solve_profile_lp(m, n, K, g->hA.data(), g->hB.data(), g->hprior.data(), prof.data(),
                                    x.data(), &v_lp);
    if (rc == 2) return fail(BSSE_ESTATE, "the simplex method did not converge");
    if (rc == 1) return fail(BSSE_EINVAL, "the profile is a best response nowhere on the simplex");
    // the segment from the program's vertex to the sweep's winner: the vertex sits on the boundary
    // of the profile's region, where fp32 rounding of x can tip a follower over to another action;
    // V is linear along the segment inside the region, so the best evaluated point is kept
    static const double eps[kPolishRows] = { 0.0, 0x1p-22, 0x1p-19, 0x1p-16, 0x1p-13, 0x1p-10, 0x1p-6, 1.0 };
    for (int e = 0; e < kPolishRows; ++e)
        for (int i = 0; i < m; ++i)
            rows[(size_t)e * m + i] = (float)((1.0 - eps[e]) * x[i] + eps[e] * (double)start[i]);
    if (!g->pol_rows) {
        // a row stride of m floats keeps 16-byte alignment whenever m % 4 == 0, as the kernels ask
        HIP_TRY(hipMalloc((void **)&g->pol_rows, (size_t)kPolishRows * m * sizeof(float)));
        HIP_TRY(hipMalloc((void **)&g->pol_v, (size_t)kPolishRows * sizeof(float)));
        HIP_TRY(hipMalloc((void **)&g->pol_br, (size_t)kPolishRows * K * sizeof(int32_t)));
    }
    HIP_TRY(hipMemcpyAsync(g->pol_rows, rows.data(), rows.size() * sizeof(float), hipMemcpyHostToDevice, g->stream));
    SweepArgs a{};
    a.X = g->pol_rows; a.count = kPolishRows; a.index_base = 0;
    a.V_out = g->pol_v; a.br_out = g->pol_br;
    HIP_TRY(launch_sweep(g, a, true));
    HIP_TRY(hipMemcpyAsync(vals.data(), g->pol_v, vals.size() * sizeof(float), hipMemcpyDeviceToHost, g->stream));
    HIP_TRY(hipMemcpyAsync(brs.data(), g->pol_br, brs.size() * sizeof(int32_t), hipMemcpyDeviceToHost, g->stream));
    HIP_TRY(hipStreamSynchronize(g->stream));
    int best = kPolishRows - 1;                          // the sweep's own winner, unless a point beats it
    for (int e = kPolishRows - 2; e >= 0; --e)
        if (vals[e] >= vals[best]) best = e;             // equal values: the point nearest the vertex
    memcpy(x_out, &rows[(size_t)best * m], (size_t)m * sizeof(float));
    res->best_value = (double)vals[best];
    res->best_index = best;
    res->n_evals = (int64_t)kPolishRows * K;
    res->n_tie_evals = 0;
    if (best_response_out) memcpy(best_response_out, &brs[(size_t)best * K], (size_t)K * sizeof(int32_t));
    if (lp_value_out) *lp_value_out = v_lp;
    return BSSE_OK;
}

extern "C" bsse_status bsse_solve_realised(bsse_game *g, const float *candidates_dev, int64_t count,
                                           int max_profiles, float *x_out, double *value_out,
                                           int32_t *profile_out, int *n_profiles_out, int *n_solved_out)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    if (!x_out || !value_out || !n_profiles_out || !n_solved_out) return fail(BSSE_EINVAL, "NULL argument");
    if (max_profiles < 1) return fail(BSSE_EINVAL, "max_profiles must be >= 1");
    bsse_status st = resolve_candidates(g, &candidates_dev, &count);
    if (st != BSSE_OK) return st;
    const int m = g->m, n = g->n, K = g->K;
    if (count == 0) return fail(BSSE_EINVAL, "no candidates");
    if ((double)count * K > (double)(1u << 27)) return fail(BSSE_EOVERFLOW, "count * K exceeds 2^27 best responses");
    const double cells = (double)m * (2.0 + (double)K * (n - 1) + m);
    if (cells > (double)(1u << 28)) return fail(BSSE_EOVERFLOW, "the program's tableau (%.3g cells) is too large", cells);
    DeviceGuard dg(g->device);
    if (!dg.ok) return fail(BSSE_EDEVICE, "hipSetDevice failed");
    DevBuf V, br;
    HIP_TRY(hipMalloc(&V.p, (size_t)count * sizeof(float)));
    HIP_TRY(hipMalloc(&br.p, (size_t)count * K * sizeof(int32_t)));
    SweepArgs a{};
    a.X = candidates_dev; a.count = count; a.index_base = 0;
    a.V_out = V.as<float>(); a.br_out = br.as<int32_t>();
    HIP_TRY(launch_sweep(g, a, true));
    std::vector<float> hv;
    std::vector<int32_t> hb;
    std::vector<int64_t> order;
    try {
        hv.resize((size_t)count); hb.resize((size_t)count * K); order.resize((size_t)count);
    } catch (...) { return fail(BSSE_ENOMEM, "host allocation failed"); }
    HIP_TRY(hipMemcpyAsync(hv.data(), V.p, hv.size() * sizeof(float), hipMemcpyDeviceToHost, g->stream));
    HIP_TRY(hipMemcpyAsync(hb.data(), br.p, hb.size() * sizeof(int32_t), hipMemcpyDeviceToHost, g->stream));
    HIP_TRY(hipStreamSynchronize(g->stream));
    // distinct profiles, each with the best value a candidate reached under it: sort the candidates
    // by profile (then value descending) and take the head of every run
    for (int64_t c = 0; c < count; ++c) order[(size_t)c] = c;
    auto prof_less = [&](int64_t x, int64_t y) {
        const int cmp = memcmp(&hb[(size_t)x * K], &hb[(size_t)y * K], (size_t)K * sizeof(int32_t));
        if (cmp != 0) return cmp < 0;
        if (hv[(size_t)x] != hv[(size_t)y]) return hv[(size_t)x] > hv[(size_t)y];
        return x < y;
    };
    std::sort(order.begin(), order.end(), prof_less);
    std::vector<int64_t> heads;
    for (int64_t i = 0; i < count; ++i)
        if (i == 0 || memcmp(&hb[(size_t)order[(size_t)i] * K], &hb[(size_t)order[(size_t)i - 1] * K],
                             (size_t)K * sizeof(int32_t)) != 0)
            heads.push_back(order[(size_t)i]);
    // most promising first: by the best swept value under the profile
    std::sort(heads.begin(), heads.end(), [&](int64_t x, int64_t y) {
        return hv[(size_t)x] != hv[(size_t)y] ? hv[(size_t)x] > hv[(size_t)y] : x < y;
    });
    *n_profiles_out = (int)(heads.size() > 0x7FFFFFFF ? 0x7FFFFFFF : heads.size());
    const size_t todo = heads.size() < (size_t)max_profiles ? heads.size() : (size_t)max_profiles;
    std::vector<double> x((size_t)m), xbest((size_t)m);
    double vbest = 0.0;
    int64_t cbest = -1;
    for (size_t i = 0; i < todo; ++i) {
        double v = 0.0;
        const int rc = solve_profile_lp(m, n, K, g->hA.data(), g->hB.data(), g->hprior.data(),
                                        &hb[(size_t)heads[i] * K], x.data(), &v);
        if (rc == 2) return fail(BSSE_ESTATE, "the simplex method did not converge");
        if (rc == 1) continue;        // realised under rounded operands only (bf16 storage)
        if (cbest < 0 || v > vbest) { vbest = v; cbest = heads[i]; xbest = x; }
    }
    *n_solved_out = (int)todo;
    if (cbest < 0) return fail(BSSE_ESTATE, "no realised profile has a feasible program");
    for (int i = 0; i < m; ++i) x_out[i] = (float)xbest[(size_t)i];
    *value_out = vbest;
    if (profile_out) memcpy(profile_out, &hb[(size_t)cbest * K], (size_t)K * sizeof(int32_t));
    return BSSE_OK;
}

// ------------------------------------------------------------------------------- timing
extern "C" bsse_status bsse_set_timing(bsse_game *g, int enabled)
{
    g_err[0] = 0;
    if (!g) return fail(BSSE_EINVAL, "game is NULL");
    DeviceGuard dg(g->device);
    bsse_status st0 = sync_all(g);
    if (st0 != BSSE_OK) return st0;
    for (hipEvent_t e : g->ev) g->ev_pool.push_back(e);
    g->ev.clear();
    g->timed_ms = 0.0; g->timed_launches = 0;
    g->timing = enabled != 0;
    return BSSE_OK;
}

extern "C" bsse_status bsse_get_timing(bsse_game *g, double *kernel_ms_out, int64_t *launches_out)
{
    g_err[0] = 0;
    if (!g || !kernel_ms_out || !launches_out) return fail(BSSE_EINVAL, "NULL argument");
    DeviceGuard dg(g->device);
    bsse_status st = sync_all(g);
    if (st != BSSE_OK) return st;
    st = drain_timing(g);
    if (st != BSSE_OK) return st;
    *kernel_ms_out = g->timed_ms;
    *launches_out = g->timed_launches;
    return BSSE_OK;
}
