// Fused sweep, matrix-core paths (steps 2-5): fp32 MFMA 32x32x2 and bf16 MFMA 32x32x16 with
// fp32 accumulation.
//
// The follower step is the skinny product  U^T = Bcat^T * X^T  with Bcat^T = all (type, action)
// rows [K*n][m] and X^T = [m][candidates]; U is never written.  The product is oriented so
// that a 32x32 MFMA tile has 32 (type, action) rows as its M dimension and 32 candidates as
// its N dimension: in the accumulator layout every lane then owns ONE candidate (column
// lane%32) and 16 of the tile's 32 rows (rows 8*(r/4) + 4*(lane/32) + r%4 for register r), so
// the arg-max over follower actions runs down a lane's own registers and needs a single
// exchange with the partner lane (lane ^ 32) per (candidate, type).
//
// Contraction index.  Lane half h = lane/32 supplies the k-slots of its half in both MFMA
// operands; this kernel maps them to leader actions i = h*MP/2 + slot, so each lane keeps a
// contiguous half of its candidate's row in registers for the whole pass over types, and the
// same registers serve the leader-payoff dot product  x . A_t[:, j*]  (each lane sums its
// half, the partner adds the other).  Payoffs are pre-packed on the host in exactly the
// per-lane fragment order, so staging a row tile into LDS is a flat copy and the operand
// reads are conflict-free.
//
// Ties.  The streaming arg-max keeps, per lane, (best value, its action) with a strict ">"
// in ascending action order, and a wave-wide bit mask (scalar registers) that records whether
// the current best has been met again exactly.  Only if some candidate of the tile ends a
// type with that bit set (or ties with its partner lane) does the wavefront take the
// second pass for that type, which recomputes the same MFMA tiles (bit-identical) and walks
// the exact maximisers in ascending action order comparing leader payoffs.
#include "bsse_internal.h"
#include <limits.h>
#include <stdlib.h>
#include <string.h>

namespace bsse {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned bf16_bits_rne(float v)
{
    unsigned b = __float_as_uint(v);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return b >> 16;
}

// ------------------------------------------------------------------------------------------
// Per-dtype pieces.  HALF = MP/2 leader actions per lane; a "fragment" is what one lane feeds
// to one MFMA.
template <typename T, int MP> struct Path;

template <int MP> struct Path<float, MP> {
    static constexpr int KSTEPS = MP / 2;      // 32x32x2: one k-slot per lane half
    static constexpr int HALF = MP / 2;
    typedef float frag;                        // one fp32 per lane per MFMA
    typedef float xreg;                        // register holding candidate components
    static constexpr int XREGS = HALF;
    static constexpr int FRAG_BYTES = 4;

    __device__ static __forceinline__ f32x16 mfma(frag a, const xreg *x, int s, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, x[s], c, 0, 0, 0);
    }
    // x registers from HALF fp32 values
    __device__ static __forceinline__ void pack_x(const float *v, xreg *x)
    {
#pragma unroll
        for (int e = 0; e < HALF; ++e) x[e] = v[e];
    }
    // sum over this lane's half of x[i] * col[i]; col points at the lane's half of the column
    __device__ static __forceinline__ float half_dot(const xreg *x, const void *col)
    {
        const float *c = (const float *)col;
        float l = 0.0f;
        if constexpr (HALF % 4 == 0) {
#pragma unroll
            for (int e = 0; e < HALF; e += 4) {
                const f32x4 v = *(const f32x4 *)(c + e);
                l = fmaf(x[e], v[0], l); l = fmaf(x[e + 1], v[1], l);
                l = fmaf(x[e + 2], v[2], l); l = fmaf(x[e + 3], v[3], l);
            }
        } else {
#pragma unroll
            for (int e = 0; e < HALF; ++e) l = fmaf(x[e], c[e], l);
        }
        return l;
    }
};

template <int MP> struct Path<__bf16, MP> {
    static_assert(MP % 16 == 0, "bf16 path needs m_pad % 16 == 0");
    static constexpr int KSTEPS = MP / 16;     // 32x32x16: eight k-slots per lane half
    static constexpr int HALF = MP / 2;
    typedef u32x4 frag;                        // eight bf16 per lane per MFMA
    typedef unsigned xreg;                     // two bf16 per register
    static constexpr int XREGS = HALF / 2;
    static constexpr int FRAG_BYTES = 16;

    __device__ static __forceinline__ f32x16 mfma(frag a, const xreg *x, int s, f32x16 c)
    {
        u32x4 b = { x[4 * s], x[4 * s + 1], x[4 * s + 2], x[4 * s + 3] };
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    __device__ static __forceinline__ void pack_x(const float *v, xreg *x)
    {
#pragma unroll
        for (int e = 0; e < HALF; e += 2)
            x[e / 2] = bf16_bits_rne(v[e]) | (bf16_bits_rne(v[e + 1]) << 16);
    }
    __device__ static __forceinline__ float half_dot(const xreg *x, const void *col)
    {
        // HIP's uint4 (a struct), not an ext_vector: bit-casting an element extracted from a
        // clang vector to a bf16 pair was seen to reuse element 0 for all four lanes of the load
        const uint4 *c = (const uint4 *)col;
        float l = 0.0f;
#pragma unroll
        for (int e = 0; e < XREGS; e += 4) {
            const uint4 v = c[e / 4];
            l = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, x[e]),
                                                __builtin_bit_cast(bf16x2, v.x), l, false);
            l = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, x[e + 1]),
                                                __builtin_bit_cast(bf16x2, v.y), l, false);
            l = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, x[e + 2]),
                                                __builtin_bit_cast(bf16x2, v.z), l, false);
            l = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, x[e + 3]),
                                                __builtin_bit_cast(bf16x2, v.w), l, false);
        }
        return l;
    }
};

// Row of a 32x32 accumulator tile held in register r, without the lane-half term 4*(lane/32).
__device__ __host__ constexpr int acc_row_base(int r) { return 8 * (r / 4) + (r % 4); }

// ------------------------------------------------------------------------------------------
// T: float | __bf16.  MP: padded m.  N: follower actions (8, 16 or a multiple of 32).
// NT: 32-candidate tiles per wavefront.  WAVES: wavefronts per workgroup.
// STAGE_TILES: 32-row tiles of packed follower payoffs per LDS stage.
template <typename T, int MP, int N, int NT, int WAVES, int STAGE_TILES>
__global__ void __launch_bounds__(WAVES * 64)
sweep_mfma_kernel(GameView g, SweepArgs a, int row_tiles)
{
    typedef Path<T, MP> P;
    typedef typename P::frag frag;
    typedef typename P::xreg xreg;
    constexpr int KS = P::KSTEPS, HALF = P::HALF;
    constexpr int TPG = N >= 32 ? N / 32 : 1;          // row tiles per group of whole types
    constexpr int TYPES = N >= 32 ? 1 : 32 / N;        // types per group
    static_assert(N == 8 || N == 16 || N % 32 == 0, "unsupported action count");
    static_assert(STAGE_TILES % TPG == 0 || TPG % STAGE_TILES == 0, "stage/group mismatch");
    constexpr int TILE_FRAGS = KS * 64;                 // fragments per row tile
    constexpr int STAGE_FRAGS = STAGE_TILES * TILE_FRAGS;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    frag *stage = reinterpret_cast<frag *>(smem);
    __shared__ float red_v[WAVES];
    __shared__ long long red_i[WAVES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, col = lane & 31;
    const int m = g.m, K = g.K;
    const frag *Bpack = reinterpret_cast<const frag *>(g.Bpack);
    const unsigned char *ATpack = reinterpret_cast<const unsigned char *>(g.ATpack);
    const long long wave_base = ((long long)blockIdx.x * WAVES + wave) * (NT * 32);

    // ---- candidate rows into registers: lane (col, h) keeps x[c][h*HALF .. h*HALF+HALF)
    xreg x[NT][P::XREGS];
    unsigned long long valid_pairs[NT];       // bit l set iff lane l's candidate exists
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        const long long c = wave_base + ct * 32 + col;
        const bool ok = c < a.count;
        float v[HALF];
        const float *row = a.X + (ok ? c : 0) * (long long)m + h * HALF;
        if (m == MP && HALF % 4 == 0 && ((uintptr_t)a.X & 15) == 0) {
#pragma unroll
            for (int e = 0; e < HALF; e += 4) {
                f32x4 q = ok ? *(const f32x4 *)(row + e) : f32x4{ 0, 0, 0, 0 };
                v[e] = q[0]; v[e + 1] = q[1]; v[e + 2] = q[2]; v[e + 3] = q[3];
            }
        } else {
#pragma unroll
            for (int e = 0; e < HALF; ++e) v[e] = (ok && h * HALF + e < m) ? row[e] : 0.0f;
        }
        P::pack_x(v, x[ct]);
        valid_pairs[ct] = __builtin_amdgcn_ballot_w64(ok);
    }

    float V[NT];
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) V[ct] = 0.0f;
    unsigned tie_count = 0;                   // wave-uniform

    // streaming arg-max state of the current group
    float best[NT][TYPES];
    int bidx[NT][TYPES];
    unsigned long long tie[NT][TYPES];

    auto reset_state = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int ti = 0; ti < TYPES; ++ti) { best[ct][ti] = -INFINITY; bidx[ct][ti] = 0; tie[ct][ti] = 0ull; }
    };

    // one 32-row tile (index tt inside its group) against all NT candidate tiles
    auto tile_pass = [&](const frag *afrags, int tt) __attribute__((always_inline)) {
        f32x16 acc[NT];
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ct][r] = 0.0f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const frag af = afrags[s * 64 + lane];
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) acc[ct] = P::mfma(af, x[ct], s, acc[ct]);
        }
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rb = tt * 32 + acc_row_base(r);      // row in group, minus 4h
                const int ti = N >= 32 ? 0 : rb / N;           // rb and rb+4 share a type (N % 8 == 0)
                const int jc = N >= 32 ? rb : rb % N;          // action, minus 4h
                const float u = acc[ct][r];
                const bool gt = u > best[ct][ti];
                const unsigned long long mgt = __builtin_amdgcn_ballot_w64(gt);
                const unsigned long long meq = __builtin_amdgcn_ballot_w64(u == best[ct][ti]);
                best[ct][ti] = gt ? u : best[ct][ti];
                bidx[ct][ti] = gt ? jc : bidx[ct][ti];
                tie[ct][ti] = (tie[ct][ti] & ~mgt) | meq;
            }
    };

    // second pass for one (candidate tile, type): exact maximisers in ascending action order,
    // leader payoff decides, then the lower action.  Reads fragments from global memory.
    auto second_pass = [&](int ct, int group, int ti, int t, float ubest, unsigned tied32,
                           float &l_out, int &j_out) __attribute__((always_inline)) {
        float lbest = 0.0f;
        int jbest = 0;
        bool has = false;
        const unsigned char *ATt = ATpack + (size_t)t * N * MP * sizeof(T);
#pragma unroll 1
        for (int tt = 0; tt < TPG; ++tt) {
            const frag *afrags = Bpack + ((size_t)group * TPG + tt) * TILE_FRAGS;
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
            for (int s = 0; s < KS; ++s) acc = P::mfma(afrags[s * 64 + lane], x[ct], s, acc);
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        const int r = 4 * q + rr;
                        const int rb = tt * 32 + acc_row_base(r);
                        if (N < 32 && rb / N != ti) continue;
                        const int j = (N >= 32 ? rb : rb % N) + 4 * hh;
                        const unsigned long long meq = __builtin_amdgcn_ballot_w64(acc[r] == ubest);
                        const unsigned hit = (unsigned)(hh ? (meq >> 32) : meq) & tied32;
                        if (hit == 0u) continue;                       // wave-uniform
                        float l = P::half_dot(x[ct], ATt + ((size_t)j * MP + h * HALF) * sizeof(T));
                        l += __shfl_xor(l, 32, 64);
                        const bool mine = (hit >> col) & 1u;
                        if (mine && (!has || l > lbest)) { lbest = l; jbest = j; has = true; }
                    }
        }
        if (has) { l_out = lbest; j_out = jbest; }
    };

    // close the types of one finished group
    auto finish_group = [&](int group) __attribute__((always_inline)) {
#pragma unroll
        for (int ti = 0; ti < TYPES; ++ti) {
            const int t = group * TYPES + ti;
            if (t >= K) break;                                          // padded type rows
            const unsigned char *ATt = ATpack + (size_t)t * N * MP * sizeof(T);
            const float pt = g.prior[t];
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) {
                const float mine = best[ct][ti];
                const int jmine = bidx[ct][ti] + 4 * h;
                const float other = __shfl_xor(mine, 32, 64);
                const int jother = __shfl_xor(jmine, 32, 64);
                const bool take = other > mine || (other == mine && jother < jmine);
                const unsigned long long mtake = __builtin_amdgcn_ballot_w64(take);
                const unsigned long long mcross = __builtin_amdgcn_ballot_w64(other == mine);
                const unsigned long long tm = tie[ct][ti];
                const unsigned long long trot = (tm >> 32) | (tm << 32);
                const unsigned long long tfin = ((tm & ~mtake) | (trot & mtake) | mcross) & valid_pairs[ct];
                const float ubest = take ? other : mine;
                int jstar = take ? jother : jmine;
                float l = P::half_dot(x[ct], ATt + ((size_t)jstar * MP + h * HALF) * sizeof(T));
                l += __shfl_xor(l, 32, 64);
                const unsigned tied32 = (unsigned)tfin | (unsigned)(tfin >> 32);
                if (tied32 != 0u) {                                     // wave-uniform, rare
                    second_pass(ct, group, ti, t, ubest, tied32, l, jstar);
                    tie_count += __builtin_popcount(tied32);
                }
                V[ct] = fmaf(pt, l, V[ct]);
                if (a.br_out) {
                    const long long c = wave_base + ct * 32 + col;
                    if (h == 0 && c < a.count) a.br_out[c * K + t] = jstar;
                }
            }
        }
    };

    auto load_stage = [&](int first_tile, int ntiles) __attribute__((always_inline)) {
        // flat copy of ntiles packed row tiles; all wavefronts of the workgroup take part
        const frag *src = Bpack + (size_t)first_tile * TILE_FRAGS;
        __syncthreads();                       // everyone is done with the previous stage
        for (int e = tid; e < ntiles * TILE_FRAGS; e += WAVES * 64) stage[e] = src[e];
        __syncthreads();
    };

    const int groups = row_tiles / TPG;
    if constexpr (STAGE_TILES >= TPG) {
        constexpr int GPS = STAGE_TILES / TPG;                          // groups per stage
#pragma unroll 1
        for (int g0 = 0; g0 < groups; g0 += GPS) {
            const int ng = groups - g0 < GPS ? groups - g0 : GPS;
            load_stage(g0 * TPG, ng * TPG);
#pragma unroll 1
            for (int gi = 0; gi < ng; ++gi) {
                reset_state();
#pragma unroll
                for (int tt = 0; tt < TPG; ++tt) tile_pass(stage + (gi * TPG + tt) * TILE_FRAGS, tt);
                finish_group(g0 + gi);
            }
        }
    } else {
        constexpr int SPG = TPG / STAGE_TILES;                          // stages per group
#pragma unroll 1
        for (int gr = 0; gr < groups; ++gr) {
            reset_state();
#pragma unroll
            for (int ss = 0; ss < SPG; ++ss) {
                load_stage(gr * TPG + ss * STAGE_TILES, STAGE_TILES);
#pragma unroll
                for (int t2 = 0; t2 < STAGE_TILES; ++t2)
                    tile_pass(stage + t2 * TILE_FRAGS, ss * STAGE_TILES + t2);
            }
            finish_group(gr);
        }
    }
    (void)STAGE_FRAGS;

    // ---- outputs
    if (a.V_out) {
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            const long long c = wave_base + ct * 32 + col;
            float v = V[ct];
            if (!(v == v)) v = -INFINITY;
            if (h == 0 && c < a.count) a.V_out[c] = v;
        }
    }
    if (a.blk_v) {
        float bv = -INFINITY;
        long long bi = LLONG_MAX;
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            const long long c = wave_base + ct * 32 + col;
            float v = V[ct];
            if (!(v == v)) v = -INFINITY;
            if (c < a.count && (v > bv || (v == bv && a.index_base + c < bi))) { bv = v; bi = a.index_base + c; }
        }
#pragma unroll
        for (int d = 16; d >= 1; d >>= 1) {          // both lane halves hold the same values
            const float ov = __shfl_xor(bv, d, 64);
            const long long oi = __shfl_xor(bi, d, 64);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        if (lane == 0) { red_v[wave] = bv; red_i[wave] = bi; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < WAVES; ++w)
                if (red_v[w] > bv || (red_v[w] == bv && red_i[w] < bi)) { bv = red_v[w]; bi = red_i[w]; }
            a.blk_v[blockIdx.x] = bv;
            a.blk_i[blockIdx.x] = bi;
        }
    }
    if (a.tie_counter && lane == 0 && tie_count) atomicAdd(a.tie_counter, (unsigned long long)tie_count);
}

// ------------------------------------------------------------------------------------------
// Instantiation table.
struct Variant {
    int storage, mp, n, nt, waves, stage_tiles;
    void (*kernel)(GameView, SweepArgs, int);
    int frag_bytes_per_tile;     // bytes of one packed 32-row tile
};

#define BSSE_VARIANT(T, ST, MPv, Nv, NTv, Wv, STv) \
    { ST, MPv, Nv, NTv, Wv, STv, sweep_mfma_kernel<T, MPv, Nv, NTv, Wv, STv>, 32 * MPv * (int)sizeof(T) }

const Variant kVariants[] = {
    // fp32 payoffs
    BSSE_VARIANT(float, 0, 8, 8, 4, 4, 1),
    BSSE_VARIANT(float, 0, 16, 16, 4, 4, 2),
    BSSE_VARIANT(float, 0, 32, 32, 4, 4, 16),
    BSSE_VARIANT(float, 0, 32, 64, 2, 4, 8),
    BSSE_VARIANT(float, 0, 128, 256, 2, 4, 2),
    // bf16 payoffs
    BSSE_VARIANT(__bf16, 1, 16, 32, 4, 4, 8),
    BSSE_VARIANT(__bf16, 1, 32, 16, 4, 4, 8),
    BSSE_VARIANT(__bf16, 1, 64, 128, 4, 4, 4),
};

const Variant *find_variant(int m, int n, int storage)
{
    const Variant *bestv = nullptr;
    for (const Variant &v : kVariants)
        if (v.storage == storage && v.n == n && v.mp >= m && (!bestv || v.mp < bestv->mp)) bestv = &v;
    return bestv;
}

int row_tiles_for(const Variant &v, int K)
{
    if (v.n >= 32) return K * (v.n / 32);
    const int tpt = 32 / v.n;
    return (K + tpt - 1) / tpt;
}

}  // namespace

bool mfma_supported(int m, int n, int K, int storage) { return find_variant(m, n, storage) != nullptr; }

long long mfma_num_blocks(const GameView &g, PathKind kind, long long count)
{
    const Variant *v = find_variant(g.m, g.n, kind == PATH_MFMA_BF16 ? 1 : 0);
    const long long per = (long long)v->nt * 32 * v->waves;
    return (count + per - 1) / per;
}

hipError_t launch_sweep_mfma(const GameView &g, PathKind kind, const SweepArgs &a, bool eval,
                             hipStream_t s)
{
    if (a.count <= 0) return hipSuccess;
    const Variant *v = find_variant(g.m, g.n, kind == PATH_MFMA_BF16 ? 1 : 0);
    if (!v) return hipErrorNotSupported;
    const long long blocks = mfma_num_blocks(g, kind, a.count);
    const size_t lds = (size_t)v->stage_tiles * v->frag_bytes_per_tile;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)v->kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(v->kernel, dim3((unsigned)blocks), dim3(v->waves * 64), lds, s, g, a,
                       row_tiles_for(*v, g.K));
    return hipGetLastError();
}

// Host packing.  Bpack: [row tile][k-step][lane 0..63][fragment], where lane = 32*h + rowInTile
// supplies leader actions i = h*MP/2 + (elements per lane)*s + e of (type, action) row
// 32*tile + rowInTile; rows past K*n and actions past m are zero.  ATpack: [K][n][MP] in
// natural action order (zero padded), so a lane's half of a column is contiguous.
void mfma_pack(int m, int n, int K, int storage, const float *A, const float *B, void **Bpack,
               size_t *Bbytes, void **ATpack, size_t *ATbytes, int *m_pad, int *n_pad)
{
    *Bpack = nullptr; *ATpack = nullptr; *Bbytes = 0; *ATbytes = 0;
    const Variant *v = find_variant(m, n, storage);
    if (!v) return;
    const int MP = v->mp, half = MP / 2;
    const int epl = storage == 1 ? 8 : 1;                  // k-slots per lane per MFMA
    const int ks = half / epl;
    const int tiles = row_tiles_for(*v, K);
    const size_t esz = storage == 1 ? 2 : 4;
    *m_pad = MP; *n_pad = n;
    *Bbytes = (size_t)tiles * 32 * MP * esz;
    *ATbytes = (size_t)K * n * MP * esz;
    unsigned char *pb = (unsigned char *)calloc(*Bbytes, 1);
    unsigned char *pa = (unsigned char *)calloc(*ATbytes, 1);
    if (!pb || !pa) { free(pb); free(pa); return; }
    auto put = [&](unsigned char *base, size_t idx, float val) {
        if (storage == 1) {
            uint32_t b; memcpy(&b, &val, 4);
            b += 0x7FFFu + ((b >> 16) & 1u);
            const uint16_t hb = (uint16_t)(b >> 16);
            memcpy(base + idx * 2, &hb, 2);
        } else {
            memcpy(base + idx * 4, &val, 4);
        }
    };
    for (int tile = 0; tile < tiles; ++tile)
        for (int s = 0; s < ks; ++s)
            for (int lane = 0; lane < 64; ++lane) {
                const int hh = lane / 32, row = tile * 32 + lane % 32;
                const int t = row / n, j = row % n;
                for (int e = 0; e < epl; ++e) {
                    const int i = hh * half + epl * s + e;
                    const float val = (t < K && i < m) ? B[((size_t)t * m + i) * n + j] : 0.0f;
                    put(pb, (((size_t)tile * ks + s) * 64 + lane) * epl + e, val);
                }
            }
    for (int t = 0; t < K; ++t)
        for (int j = 0; j < n; ++j)
            for (int i = 0; i < m; ++i)
                put(pa, ((size_t)t * n + j) * MP + i, A[((size_t)t * m + i) * n + j]);
    *Bpack = pb; *ATpack = pa;
}

}  // namespace bsse
