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
// Ties.  The accumulators of a whole type stay in registers; the arg-max is a max3 chain, one
// exchange with the partner lane, then a compare pass whose sum carries both the maximising
// action and the number of maximisers.  Anything other than one maximiser per candidate sends
// the wavefront through an exact routine for that type, which recomputes the same MFMA tiles
// (bit-identical) and walks the exact maximisers in ascending action order comparing leader
// payoffs.
#include "bsse_internal.h"
#include "mfma_device.h"
#include <limits.h>
#include <stdlib.h>
#include <string.h>

namespace bsse {

namespace {

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
    template <typename BP>      // BP: byte pointer, global (generic) or LDS address space
    __device__ static __forceinline__ float half_dot(const xreg *x, BP col)
    {
        typedef typename std::conditional<std::is_same<BP, const lds_byte *>::value,
                                          const __attribute__((address_space(3))) float *, const float *>::type FP;
        typedef typename std::conditional<std::is_same<BP, const lds_byte *>::value,
                                          const __attribute__((address_space(3))) f32x4 *, const f32x4 *>::type VP;
        const FP c = (FP)col;
        float l = 0.0f;
        if constexpr (HALF % 4 == 0) {
#pragma unroll
            for (int e = 0; e < HALF; e += 4) {
                const f32x4 v = *(VP)(c + e);
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
    template <typename BP>
    __device__ static __forceinline__ float half_dot(const xreg *x, BP col)
    {
        // l += x.lo*c.lo + x.hi*c.hi on packed bf16 pairs, fp32 accumulate.  Issued as asm on
        // plain 32-bit words: going through the bf16-pair builtin, a bit-cast of an element
        // extracted from a clang vector was seen to reuse element 0 for all four words of a load.
        typedef typename std::conditional<std::is_same<BP, const lds_byte *>::value,
                                          const __attribute__((address_space(3))) u32x4 *, const u32x4 *>::type VP;
        const VP c = (VP)col;
        float l0 = 0.0f, l1 = 0.0f;
#pragma unroll
        for (int e = 0; e < XREGS; e += 4) {
            const u32x4 v = c[e / 4];
            const unsigned w0 = v[0], w1 = v[1], w2 = v[2], w3 = v[3];
            asm("v_dot2c_f32_bf16 %0, %2, %6\n\t"
                "v_dot2c_f32_bf16 %1, %3, %7\n\t"
                "v_dot2c_f32_bf16 %0, %4, %8\n\t"
                "v_dot2c_f32_bf16 %1, %5, %9\n\t"
                "s_nop 2"       // a dot result needs three wait states before another kind of
                                // vector instruction reads it; the compiler cannot see into asm
                : "+v"(l0), "+v"(l1)
                : "v"(x[e]), "v"(x[e + 1]), "v"(x[e + 2]), "v"(x[e + 3]), "v"(w0), "v"(w1), "v"(w2), "v"(w3));
        }
        const float l = l0 + l1;
        return l;
    }
    // The same sum in two steps -- the lane's half of the column into registers, then the dot
    // product -- so that a caller can put other work between the reads and their use.  Same
    // instruction sequence on the same values as half_dot, hence the same bits.
    typedef u32x4 colregs[XREGS / 4];
    __device__ static __forceinline__ void gather_half(const lds_byte *col, colregs &c)
    {
        const __attribute__((address_space(3))) u32x4 *p = (const __attribute__((address_space(3))) u32x4 *)col;
#pragma unroll
        for (int e = 0; e < XREGS / 4; ++e) c[e] = p[e];
    }
    __device__ static __forceinline__ float half_dot_regs(const xreg *x, const colregs &c)
    {
        float l0 = 0.0f, l1 = 0.0f;
#pragma unroll
        for (int e = 0; e < XREGS; e += 4) {
            const unsigned w0 = c[e / 4][0], w1 = c[e / 4][1], w2 = c[e / 4][2], w3 = c[e / 4][3];
            // (a dot result feeding the next dot needs no wait states; the three that another kind
            // of vector instruction needs follow the last group only)
            asm volatile("v_dot2c_f32_bf16 %0, %2, %6\n\t"
                         "v_dot2c_f32_bf16 %1, %3, %7\n\t"
                         "v_dot2c_f32_bf16 %0, %4, %8\n\t"
                         "v_dot2c_f32_bf16 %1, %5, %9"
                         : "+v"(l0), "+v"(l1)
                         : "v"(x[e]), "v"(x[e + 1]), "v"(x[e + 2]), "v"(x[e + 3]), "v"(w0), "v"(w1), "v"(w2), "v"(w3));
        }
        asm volatile("s_nop 2" : "+v"(l0), "+v"(l1));
        return l0 + l1;
    }
    // Two candidate tiles at once: the four accumulation chains are interleaved (a dot product
    // feeding the next one of its chain waits for it), each chain as in half_dot_regs.
    __device__ static __forceinline__ void half_dot_regs2(const xreg *xa, const colregs &ca, const xreg *xb,
                                                          const colregs &cb, float &la, float &lb)
    {
        float a0 = 0.0f, a1 = 0.0f, b0 = 0.0f, b1 = 0.0f;
#pragma unroll
        for (int e = 0; e < XREGS; e += 4) {
            const unsigned p0 = ca[e / 4][0], p1 = ca[e / 4][1], p2 = ca[e / 4][2], p3 = ca[e / 4][3];
            const unsigned q0 = cb[e / 4][0], q1 = cb[e / 4][1], q2 = cb[e / 4][2], q3 = cb[e / 4][3];
            asm volatile("v_dot2c_f32_bf16 %0, %4, %8\n\t"
                         "v_dot2c_f32_bf16 %2, %12, %16\n\t"
                         "v_dot2c_f32_bf16 %1, %5, %9\n\t"
                         "v_dot2c_f32_bf16 %3, %13, %17\n\t"
                         "v_dot2c_f32_bf16 %0, %6, %10\n\t"
                         "v_dot2c_f32_bf16 %2, %14, %18\n\t"
                         "v_dot2c_f32_bf16 %1, %7, %11\n\t"
                         "v_dot2c_f32_bf16 %3, %15, %19"
                         : "+v"(a0), "+v"(a1), "+v"(b0), "+v"(b1)
                         : "v"(xa[e]), "v"(xa[e + 1]), "v"(xa[e + 2]), "v"(xa[e + 3]), "v"(p0), "v"(p1), "v"(p2), "v"(p3),
                           "v"(xb[e]), "v"(xb[e + 1]), "v"(xb[e + 2]), "v"(xb[e + 3]), "v"(q0), "v"(q1), "v"(q2), "v"(q3));
        }
        asm volatile("s_nop 2" : "+v"(a0), "+v"(a1), "+v"(b0), "+v"(b1));
        la = a0 + a1;
        lb = b0 + b1;
    }
    // The same sum when the column holds three identical blocks (payoffs that are bf16 numbers,
    // against the three parts of x): each 16 bytes of the first block are loaded once and used
    // for all three parts, instead of gathering the same values three times.
    template <typename BP>
    __device__ static __forceinline__ float half_dot_rep3(const xreg *x, BP col)
    {
        typedef typename std::conditional<std::is_same<BP, const lds_byte *>::value,
                                          const __attribute__((address_space(3))) u32x4 *, const u32x4 *>::type VP;
        static_assert(XREGS % 12 == 0, "three blocks of whole 16-byte pieces");
        constexpr int BLOCK = XREGS / 3;
        const VP c = (VP)col;
        float l0 = 0.0f, l1 = 0.0f;
#pragma unroll
        for (int e = 0; e < BLOCK; e += 4) {
            const u32x4 v = c[e / 4];
            const unsigned w0 = v[0], w1 = v[1], w2 = v[2], w3 = v[3];
#pragma unroll
            for (int term = 0; term < 3; ++term) {
                const int b = term * BLOCK + e;
                asm("v_dot2c_f32_bf16 %0, %2, %6\n\t"
                    "v_dot2c_f32_bf16 %1, %3, %7\n\t"
                    "v_dot2c_f32_bf16 %0, %4, %8\n\t"
                    "v_dot2c_f32_bf16 %1, %5, %9\n\t"
                    "s_nop 2"
                    : "+v"(l0), "+v"(l1)
                    : "v"(x[b]), "v"(x[b + 1]), "v"(x[b + 2]), "v"(x[b + 3]), "v"(w0), "v"(w1), "v"(w2), "v"(w3));
            }
        }
        const float l = l0 + l1;
        return l;
    }
};

// ------------------------------------------------------------------------------------------
// Stage records.  The packed follower payoffs are cut into "stages" of STAGE_TILES 32-row
// tiles; when AT_LDS, the leader-payoff rows of the types a stage covers follow its tiles, so
// that one flat asynchronous copy (global_load_lds) brings everything a stage needs into LDS.
// Leader rows in LDS are padded by 16 bytes so that gathers of different rows spread over
// banks.  The record size is rounded to what one sweep of all wavefronts copies (1 KiB each).
struct Geometry {
    int tile_bytes, tpg, types, ts, ats, at_bytes, rec_bytes;
};
// terms == 6 (both operands split into bf16 parts) with leader rows in LDS: the leader rows are kept
// as plain fp32 (mp / terms values and 16 bytes of padding per action), not as parts.
// terms == 3 (payoffs that are bf16 numbers against the three parts of the candidate): the three
// blocks of a row tile's fragments would be identical, so a tile holds one block (mp / 3 slots)
// and every fragment read serves three matrix instructions.
__host__ __device__ constexpr Geometry make_geometry(int esz, int mp, int n, int stage_tiles,
                                                     int waves, bool at_lds, int terms = 1)
{
    Geometry q{};
    q.tile_bytes = 32 * (terms == 3 ? mp / 3 : mp) * esz;
    q.tpg = n >= 32 ? n / 32 : 1;
    q.types = n >= 32 ? 1 : 32 / n;
    q.ts = stage_tiles >= q.tpg ? (stage_tiles / q.tpg) * q.types : 0;     // whole types per stage
    q.ats = (terms == 6 && at_lds) ? (mp / terms + 4) * 4 / esz : mp + 16 / esz;   // in elements of esz
    q.at_bytes = at_lds ? q.ts * n * q.ats * esz : 0;
    const int unit = waves * 1024;
    q.rec_bytes = (stage_tiles * q.tile_bytes + q.at_bytes + unit - 1) / unit * unit;
    return q;
}

// dynamic LDS of sweep_wide_kernel: two fragment buffers and two leader-row buffers
__host__ __device__ constexpr int wide_lds_bytes(int esz, int mp, int n, int waves)
{
    const Geometry q = make_geometry(esz, mp, n, n / 32, waves, true);
    return 2 * (q.tpg * q.tile_bytes) + 2 * ((q.at_bytes + 1023) / 1024 * 1024);
}

typedef const void __attribute__((address_space(1))) *global_ptr;
typedef void __attribute__((address_space(3))) *lds_ptr;

// ------------------------------------------------------------------------------------------
// T: float | __bf16.  MP: padded m.  N: follower actions (8, 16 or a multiple of 32).
// NT: 32-candidate tiles per wavefront.  WAVES: wavefronts per workgroup.
// STAGE_TILES: row tiles per LDS stage.  OCC: wavefronts per SIMD the register allocation is
// held to.  AT_LDS: leader-payoff rows travel with the stage (else they are gathered from
// global memory / L2).
//
// A "group" is the set of row tiles that holds whole types: N/32 tiles of one type when
// N >= 32, one tile of 32/N types otherwise.  The accumulators of a whole group stay in
// registers (N/2 per lane and candidate tile when N >= 32), so the arg-max is two passes
// over registers: a max3 chain for the lane's maximum, one exchange with the partner lane
// for the pair's maximum, then a compare pass that adds (action + 2^16) for every register
// equal to the maximum: the sum carries the maximising action and the number of maximisers.
// Anything other than one maximiser per candidate means an exact tie somewhere in the tile
// and sends the wavefront through the exact routine for that type.
//
// Stages are double-buffered: the copy of stage s+1 is issued (asynchronously, straight into
// LDS) before the work on stage s and awaited after it, one workgroup barrier per stage.
//
// SLICED: the launch is two-dimensional and workgroup row blockIdx.y walks only its slice of the
// stages (whole groups), writing the per-type leader payoffs instead of the value; used to
// re-evaluate a few rows against many types with the whole chip.  The per-candidate instruction
// sequence does not depend on NT, OCC or SLICED, so every instantiation of a packing gives the
// same bits for the same row.
template <typename T, int MP, int N, int NT, int WAVES, int STAGE_TILES, int OCC, bool AT_LDS, int TERMS,
          bool SLICED, int PF>
__global__ void __launch_bounds__(WAVES * 64, OCC)
sweep_mfma_kernel(GameView g, SweepArgs a, int row_tiles)
{
    static_assert(TERMS == 1 || TERMS == 3 || TERMS == 6, "1 = operands as stored; 3, 6 = split fp32");
    static_assert(TERMS == 1 || std::is_same<T, __bf16>::value, "split terms run on the bf16 path");
    static_assert(MP % TERMS == 0, "MP is TERMS blocks of the padded m");
    constexpr int MP_BASE = MP / TERMS, HALF_BASE = MP_BASE / 2;
    typedef Path<T, MP> P;
    typedef typename P::frag frag;
    typedef typename P::xreg xreg;
    constexpr int KS = P::KSTEPS, HALF = P::HALF;
    constexpr Geometry G = make_geometry((int)sizeof(T), MP, N, STAGE_TILES, WAVES, AT_LDS, TERMS);
    constexpr int TPG = G.tpg, TYPES = G.types;
    static_assert(N == 8 || N == 16 || N % 32 == 0, "unsupported action count");
    static_assert(STAGE_TILES % TPG == 0 || TPG % STAGE_TILES == 0, "stage/group mismatch");
    static_assert(!AT_LDS || STAGE_TILES >= TPG, "leader rows in LDS need whole types per stage");
    constexpr int REP = TERMS == 3 ? 3 : 1;             // matrix instructions per fragment read
    constexpr int KF = KS / REP;                        // fragment k-steps per row tile
    constexpr int TILE_FRAGS = KF * 64;                 // fragments per row tile
    static_assert(PF == 0 || REP == 1, "the chunked fragment read-ahead takes one instruction per fragment");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ float red_v[WAVES];
    __shared__ long long red_i[WAVES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, col = lane & 31;
    const int m = g.m, K = g.K;
    const unsigned char *records = reinterpret_cast<const unsigned char *>(g.Bpack);
    const unsigned char *ATpack = reinterpret_cast<const unsigned char *>(g.ATpack);
    const long long wave_base = ((long long)blockIdx.x * WAVES + wave) * (NT * 32);
    const int nstages = (row_tiles + STAGE_TILES - 1) / STAGE_TILES;
    // the stages this workgroup walks: all of them, or slice blockIdx.y of them
    const int stage_begin = SLICED ? (int)blockIdx.y * a.slice_stages : 0;
    const int stage_end = SLICED && stage_begin + a.slice_stages < nstages
                              ? stage_begin + a.slice_stages : nstages;
    if (SLICED && stage_begin >= stage_end) return;                     // whole workgroup

    auto prefetch = [&](int st) __attribute__((always_inline)) {
        const unsigned char *src = records + (size_t)st * G.rec_bytes;
        unsigned char *dst = smem + (st & 1) * G.rec_bytes;
#pragma unroll
        for (int i = 0; i < G.rec_bytes / (WAVES * 1024); ++i) {
            const int chunk = i * WAVES + wave;
            __builtin_amdgcn_global_load_lds((global_ptr)(src + chunk * 1024 + lane * 16),
                                             (lds_ptr)(dst + chunk * 1024), 16, 0, 0);
        }
    };
    // own copies have landed; then everyone's have, and everyone is done with the old stage
    auto stage_sync = [&]() __attribute__((always_inline)) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    };
    prefetch(stage_begin);

    // ---- candidate rows into registers: lane (col, h) keeps its half of the leader actions,
    // x[c][h*HALF_BASE .. (h+1)*HALF_BASE); on the split path each component becomes TERMS
    // bf16 parts, laid out as TERMS blocks of HALF_BASE to match the packed payoffs
    // Split path: three bf16 parts per component are stored once each (p0, p1, p2 as blocks of
    // XB registers); the six k-slot blocks (p0,B0) (p0,B1) (p1,B0) (p0,B2) (p1,B1) (p2,B0) of the
    // packed payoffs pick them in x_mfma.  Where the leader rows are in LDS they are fp32, and
    // so is the lane's half of the candidate row that meets them (xf).
    constexpr bool LEAD_F32 = TERMS == 6 && AT_LDS;
    constexpr int XB = TERMS > 1 ? HALF_BASE / 2 : P::XREGS;            // registers per part
    constexpr int XS = TERMS > 1 ? 3 * XB : P::XREGS;                   // registers stored per tile
    constexpr int SPT = KS / TERMS;                                     // k-steps per block
    auto x_mfma = [](const frag &fr, const xreg *xc, int s, const f32x16 &c) __attribute__((always_inline)) {
        if constexpr (TERMS == 6) {
            constexpr int xsel6[6] = { 0, 0, 1, 0, 1, 2 };
            return P::mfma(fr, xc + xsel6[s / SPT] * XB + 4 * (s % SPT), 0, c);
        } else {
            return P::mfma(fr, xc, s, c);
        }
    };
    xreg x[NT][XS];
    float xf[NT][LEAD_F32 ? HALF_BASE : 1];
    unsigned valid32[NT];                     // bit c set iff candidate c of the tile exists
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        const long long c = wave_base + ct * 32 + col;
        const bool ok = c < a.count;
        float vb[HALF_BASE];
        const float *row = a.X + (ok ? c : 0) * (long long)m + h * HALF_BASE;
        if (m == MP_BASE && HALF_BASE % 4 == 0 && ((uintptr_t)a.X & 15) == 0) {
#pragma unroll
            for (int e = 0; e < HALF_BASE; e += 4) {
                f32x4 q = ok ? *(const f32x4 *)(row + e) : f32x4{ 0, 0, 0, 0 };
                vb[e] = q[0]; vb[e + 1] = q[1]; vb[e + 2] = q[2]; vb[e + 3] = q[3];
            }
        } else {
#pragma unroll
            for (int e = 0; e < HALF_BASE; ++e) vb[e] = (ok && h * HALF_BASE + e < m) ? row[e] : 0.0f;
        }
        if constexpr (TERMS == 1) {
            P::pack_x(vb, x[ct]);
        } else {
            // x = p0 + p1 + p2 with bf16 parts (the subtractions are exact in fp32)
            float v[3 * HALF_BASE];
#pragma unroll
            for (int e = 0; e < HALF_BASE; ++e) {
                float part[3];
                part[0] = __uint_as_float(bf16_bits_rne(vb[e]) << 16);
                const float r1 = vb[e] - part[0];
                part[1] = __uint_as_float(bf16_bits_rne(r1) << 16);
                const float r2 = r1 - part[1];
                part[2] = __uint_as_float(bf16_bits_rne(r2) << 16);
#pragma unroll
                for (int q = 0; q < 3; ++q) v[q * HALF_BASE + e] = part[q];
            }
#pragma unroll
            for (int e = 0; e < 3 * HALF_BASE; e += 2)
                x[ct][e / 2] = bf16_bits_rne(v[e]) | (bf16_bits_rne(v[e + 1]) << 16);
            if constexpr (LEAD_F32) {
#pragma unroll
                for (int e = 0; e < HALF_BASE; ++e) xf[ct][e] = vb[e];
            }
        }
        valid32[ct] = (unsigned)__builtin_amdgcn_ballot_w64(ok);
    }

    float V[NT];
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) V[ct] = 0.0f;
    unsigned tie_count = 0;                   // wave-uniform
    // per-register constants of the compare pass: the action a register stands for within its
    // row tile and type (lane half included) plus 2^16
    unsigned creg[16];
#pragma unroll
    for (int r = 0; r < 16; ++r)
        creg[r] = (unsigned)((N >= 32 ? acc_row_base(r) : acc_row_base(r) % N) + 4 * h) + 65536u;

    // Leader-payoff half sum over a column gathered from global memory.  With three part products
    // the column's three blocks are identical, and one is read.
    auto leader_half = [&](const xreg *xc, const unsigned char *colp) __attribute__((always_inline)) {
        if constexpr (TERMS == 3 && !AT_LDS) return P::half_dot_rep3(xc, colp);
        else return P::half_dot(xc, colp);
    };
    // fp32 leader rows (LEAD_F32): the lane's HALF_BASE components against its half of the row,
    // two fused multiply-add chains; the same sequence from LDS and from global memory.
    auto leader_half_f32 = [&](const float *xc, auto row) __attribute__((always_inline)) {
        float l0 = 0.0f, l1 = 0.0f;
#pragma unroll
        for (int e = 0; e < (LEAD_F32 ? HALF_BASE : 0); e += 4) {
            const f32x4 r = row[e / 4];
            l0 = fmaf(xc[e], r[0], l0); l1 = fmaf(xc[e + 1], r[1], l1);
            l0 = fmaf(xc[e + 2], r[2], l0); l1 = fmaf(xc[e + 3], r[3], l1);
        }
        return l0 + l1;
    };
    // Exact routine for one (candidate tile, type): recomputes the type's tiles one at a time
    // from the packed records in global memory (same instruction sequence, hence the same
    // bits), visits the exact maximisers in ascending action order, lets the leader's payoff
    // decide and then the lower action.
    auto exact_type = [&](int ct, int group, int ti, int t, float gmax, float &l_out,
                          int &j_out) __attribute__((always_inline)) {
        float lbest = 0.0f;
        int jbest = 0, nmatch = 0;
        const unsigned char *ATt = ATpack + (size_t)t * N * MP * sizeof(T);
#pragma unroll 1
        for (int tt = 0; tt < TPG; ++tt) {
            const int gt = group * TPG + tt;
            const frag *afrags = reinterpret_cast<const frag *>(
                records + (size_t)(gt / STAGE_TILES) * G.rec_bytes + (size_t)(gt % STAGE_TILES) * G.tile_bytes);
            f32x16 acc1;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc1[r] = 0.0f;
#pragma unroll
            for (int s = 0; s < KF; ++s) {
                const frag af = afrags[s * 64 + lane];
#pragma unroll
                for (int q = 0; q < REP; ++q) acc1 = x_mfma(af, x[ct], q * KF + s, acc1);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        const int r = 4 * q + rr;
                        const int rb = acc_row_base(r);
                        if (N < 32 && rb / N != ti) continue;
                        const int j = (N >= 32 ? tt * 32 + rb : rb % N) + 4 * hh;
                        const unsigned long long meq = __builtin_amdgcn_ballot_w64(acc1[r] == gmax);
                        const unsigned hit = (unsigned)(hh ? (meq >> 32) : meq) & valid32[ct];
                        if (hit == 0u) continue;                       // wave-uniform
                        float lh;
                        if constexpr (LEAD_F32)
                            lh = leader_half_f32(xf[ct], reinterpret_cast<const f32x4 *>(
                                     reinterpret_cast<const float *>(ATpack) + ((size_t)t * N + j) * MP_BASE + h * HALF_BASE));
                        else
                            lh = leader_half(x[ct], ATt + ((size_t)j * MP + h * HALF) * sizeof(T));
                        const float l = pair_sum(lh);
                        if ((hit >> col) & 1u) {
                            if (nmatch == 0 || l > lbest) { lbest = l; jbest = j; }
                            ++nmatch;
                        }
                    }
        }
        l_out = lbest; j_out = jbest;
        tie_count += __builtin_popcount((unsigned)__builtin_amdgcn_ballot_w64(nmatch >= 2));
    };

    // accumulators of the current group, all NT candidate tiles
    f32x16 acc[NT][TPG];
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int tt = 0; tt < TPG; ++tt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[ct][tt][r] = 0.0f;
    };
    // MFMAs of NTILES consecutive row tiles (fragments in LDS at `base`; tt0 = index of the first
    // one within the group) against all NT candidate tiles.  The fragment reads are software-
    // pipelined in chunks of PF k-steps where that was measured to pay (the wide bf16 game): the
    // reads of chunk q+1 are issued before the MFMAs of chunk q, so the LDS latency runs under the
    // matrix pipe instead of in front of it.
    auto mfma_run = [&](const frag *base, auto ntiles_c, auto tt0_c) __attribute__((always_inline)) {
        constexpr int NTILES = decltype(ntiles_c)::value, TT0 = decltype(tt0_c)::value;
        if constexpr (PF == 0) {               // reads where they are used; the compiler schedules
#pragma unroll
            for (int tt = 0; tt < NTILES; ++tt)
#pragma unroll
                for (int ks = 0; ks < KF; ++ks) {
                    const frag af = base[(size_t)tt * TILE_FRAGS + (size_t)ks * 64 + lane];
#pragma unroll
                    for (int q = 0; q < REP; ++q)
#pragma unroll
                        for (int ct = 0; ct < NT; ++ct)
                            acc[ct][TT0 + tt] = x_mfma(af, x[ct], q * KF + ks, acc[ct][TT0 + tt]);
                }
            return;
        }
        static_assert(PF == 0 || KS % (PF ? PF : 1) == 0, "fragment chunk must divide the k-steps of a tile");
        constexpr int C = PF ? PF : 1;
        constexpr int NCH = NTILES * KS / C;
        frag fb[2][C];
        const frag *lane_base = base + lane;
#pragma unroll
        for (int e = 0; e < C; ++e) fb[0][e] = lane_base[(size_t)e * 64];
        static_for<0, NCH, 1>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            if constexpr (q + 1 < NCH) {
#pragma unroll
                for (int e = 0; e < C; ++e) {
                    constexpr int f0 = (q + 1) * C;
                    const int f = f0 + e;                                    // flat (tile, k-step)
                    fb[(q + 1) & 1][e] = lane_base[(size_t)(f / KS) * TILE_FRAGS + (size_t)(f % KS) * 64];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            static_for<0, C, 1>([&](auto ec) {
                constexpr int f = q * C + decltype(ec)::value;
                constexpr int tt = TT0 + f / KS, ks = f % KS;
#pragma unroll
                for (int ct = 0; ct < NT; ++ct) acc[ct][tt] = x_mfma(fb[q & 1][decltype(ec)::value], x[ct], ks, acc[ct][tt]);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    // second half of a type's epilogue: leader payoff at the best response (fast path: one row
    // gather and a dot product; otherwise the exact routine), value accumulation, outputs
    auto leader_part = [&](int group, int ti, int t, float pt, const lds_byte *at_lds, const float *gmax,
                           const int *jstar, const bool *clean) __attribute__((always_inline)) {
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            float l;
            int js = jstar[ct];
            if (clean[ct]) {
                float part;
                if constexpr (LEAD_F32)
                    part = leader_half_f32(xf[ct], (const __attribute__((address_space(3))) f32x4 *)(
                               at_lds + (unsigned)(((ti * N + js) * G.ats) * sizeof(T) + h * HALF_BASE * sizeof(float))));
                else if constexpr (AT_LDS)
                    part = P::half_dot(x[ct], at_lds + (unsigned)(((ti * N + js) * G.ats + h * HALF) * sizeof(T)));
                else
                    part = leader_half(x[ct], ATpack + (((size_t)t * N + js) * MP + h * HALF) * sizeof(T));
                l = pair_sum(part);
            } else {
                exact_type(ct, group, ti, t, gmax[ct], l, js);
            }
            V[ct] = fmaf(pt, l, V[ct]);
            if (a.br_out) {
                const long long c = wave_base + ct * 32 + col;
                if (h == 0 && c < a.count) a.br_out[c * K + t] = js;
            }
            if constexpr (SLICED) {
                const long long c = wave_base + ct * 32 + col;
                if (h == 0 && c < a.count) a.l_out[c * K + t] = l;
            }
        }
    };
    // per-type epilogue of a finished group; at_lds = LDS rows of the group's first type
    auto epilogue = [&](int group, const lds_byte *at_lds) __attribute__((always_inline)) {
        // The asm blocks below read the accumulators, and the compiler's hazard handling does not
        // look into inline asm: the wait states a vector read of a fresh MFMA result needs (passes
        // + 3: 11 for the 8-pass bf16 MFMA, 19 for the 16-pass fp32 one) are put here explicitly.
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_nop 15");
        if constexpr (std::is_same<T, float>::value) asm volatile("s_nop 3");
        static_for<0, TYPES, 1>([&](auto tic) {
            constexpr int ti = decltype(tic)::value;
            const int t = group * TYPES + ti;
            if (t >= K) return;                                         // padded type rows
            const float pt = g.prior[t];
            float gmax[NT];
            int jstar[NT];
            bool clean[NT];
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) {
                // lane maximum over this type's registers
                float pm = -INFINITY;
                unsigned total = 0u, tile_tie = 0u;       // tile_tie: wave-uniform column mask
                float gm;
                if constexpr (N >= 32) {
                    // whole row tiles belong to the type: one asm block per 16 registers for the
                    // maximum and one for the compare pass
                    float u[TPG][16];
#pragma unroll
                    for (int tt = 0; tt < TPG; ++tt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) u[tt][r] = acc[ct][tt][r];
                    if constexpr (TPG == 1) {
                        pm = vmax_chain16(pm, u[0]);
                        gm = pair_max(pm);
                        match8(u[0], gm, creg, total);
                        match8(u[0] + 8, gm, creg + 8, total);
                    } else {
                        // Lane maximum per row tile (tile tt goes with tile tt + TPG/2: two
                        // independent instruction streams), then over the tiles.
                        constexpr int HT = TPG / 2;
                        float pmt[TPG];
#pragma unroll
                        for (int k = 0; k < TPG; ++k) pmt[k] = -INFINITY;
                        static_for<0, HT, 1>([&](auto ttc) {
                            constexpr int tt = decltype(ttc)::value;
                            vmax_chain16x2(pmt[tt], u[tt], pmt[tt + HT], u[tt + HT]);
                        });
                        pm = pmt[0];
#pragma unroll
                        for (int k = 1; k + 1 < TPG; k += 2) pm = vmax3(pm, pmt[k], pmt[k + 1]);
                        pm = vmax2(pm, pmt[TPG - 1]);
                        gm = pair_max(pm);
                        // Only a tile whose maximum is the pair's maximum can hold a maximiser.
                        // Two such tiles in one lane are a tie (exact routine); otherwise the
                        // tile's sixteen registers are selected (a tournament of conditional
                        // moves, (TPG-1)*16 of them) and the compare pass runs on those alone:
                        // (TPG-1)*16 + 32 instructions instead of TPG*32.
                        bool e[TPG];
                        unsigned tile[TPG];
                        unsigned long long seen = 0ull, dup = 0ull;
#pragma unroll
                        for (int k = 0; k < TPG; ++k) {
                            e[k] = pmt[k] == gm;
                            tile[k] = (unsigned)k;
                            const unsigned long long mk = __builtin_amdgcn_ballot_w64(e[k]);
                            dup |= seen & mk;
                            seen |= mk;
                        }
                        tile_tie |= (unsigned)(dup | (dup >> 32));
#pragma unroll
                        for (int nn = TPG; nn > 1; nn >>= 1)
#pragma unroll
                            for (int j = 0; j < nn / 2; ++j) {
#pragma unroll
                                for (int r = 0; r < 16; ++r) u[j][r] = e[2 * j + 1] ? u[2 * j + 1][r] : u[2 * j][r];
                                tile[j] = e[2 * j + 1] ? tile[2 * j + 1] : tile[2 * j];
                                e[j] = e[2 * j] || e[2 * j + 1];
                            }
                        // compare pass as a bitmap: bit 15 - r set iff register r is a maximiser
                        const unsigned w = bitmap16_split(u[0], gm);
                        const unsigned cnt = (unsigned)__builtin_popcount(w);
                        const unsigned r = ffbh(w) - 16u;
                        // action = 32 * tile + row(register) + 4h
                        const unsigned act = (tile[0] << 5) | ((r & 0xCu) << 1) | (r & 3u) | (4u * h);
                        total = cnt ? (cnt << 16) | act : 0u;
                    }
                } else {
                    float pend[2];
                    int np = 0;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        if (acc_row_base(r) / N != ti) continue;
                        pend[np++] = acc[ct][0][r];
                        if (np == 2) { pm = vmax3(pm, pend[0], pend[1]); np = 0; }
                    }
                    if (np == 1) pm = vmax2(pm, pend[0]);
                    gm = pair_max(pm);
                    // compare pass over the type's registers of the tile
                    static_for<0, 4, 1>([&](auto qc) {
                        constexpr int r = 4 * decltype(qc)::value;
                        if constexpr (acc_row_base(r) / N == ti)
                            match4(acc[ct][0][r], acc[ct][0][r + 1], acc[ct][0][r + 2], acc[ct][0][r + 3],
                                   gm, creg[r], creg[r + 1], creg[r + 2], creg[r + 3], total);
                    });
                }
                const unsigned pair = pair_add_u32(total);
                gmax[ct] = gm;
                jstar[ct] = (int)(pair & 0xFFFFu);
                const unsigned multi = (unsigned)__builtin_amdgcn_ballot_w64((pair >> 16) != 1u) | tile_tie;
                clean[ct] = (multi & valid32[ct]) == 0u && valid32[ct] == 0xFFFFFFFFu;   // wave-uniform
            }
            leader_part(group, ti, t, pt, at_lds, gmax, jstar, clean);
        });
    };

    stage_sync();                              // the first stage is in LDS
    const int groups = row_tiles / TPG;
    // Two roles where the epilogue reads nothing from LDS (leader rows gathered from global memory),
    // a stage holds whole types and one workgroup fills the compute unit: the late half of the
    // wavefronts passes the barrier that ends a stage BEFORE the stage's last epilogue, the early half
    // after it, so that behind every barrier the two wavefronts of a SIMD are one epilogue apart
    // -- one on the matrix pipe, one on the vector unit -- instead of wanting the same unit at the
    // same time (measured on the m=128 n=256 three-term variant: 4 %; with a barrier per row tile
    // the late half held the early half up instead, and on the wide bf16 kernel it gained nothing).
    constexpr bool ROLES = !AT_LDS && !SLICED && WAVES == 8 && STAGE_TILES >= TPG;
    const bool late = ROLES && wave >= WAVES / 2;
    if constexpr (STAGE_TILES >= TPG) {
        constexpr int GPS = STAGE_TILES / TPG;                          // groups per stage
#pragma unroll 1
        for (int st = stage_begin; st < stage_end; ++st) {
            if (st + 1 < stage_end) prefetch(st + 1);
            const unsigned char *buf = smem + (st & 1) * G.rec_bytes;
            const frag *tiles = reinterpret_cast<const frag *>(buf);
            const int g0 = st * GPS;
            const int ng = groups - g0 < GPS ? groups - g0 : GPS;
#pragma unroll 1
            for (int gi = 0; gi < ng; ++gi) {
                zero_acc();
                mfma_run(tiles + (size_t)(gi * TPG) * TILE_FRAGS, std::integral_constant<int, TPG>{},
                         std::integral_constant<int, 0>{});
                if (ROLES && late && gi == ng - 1) stage_sync();
                epilogue(g0 + gi, (const lds_byte *)buf + (unsigned)(STAGE_TILES * G.tile_bytes + gi * TYPES * N * G.ats * sizeof(T)));
            }
            if (!(ROLES && late) || ng <= 0) stage_sync();      // (every wavefront: one barrier per stage)
        }
    } else {
        constexpr int SPG = TPG / STAGE_TILES;                          // stages per group
        int st = stage_begin;                                           // a multiple of SPG
        const int group_end = stage_end / SPG < groups ? stage_end / SPG : groups;
#pragma unroll 1
        for (int gr = stage_begin / SPG; gr < group_end; ++gr) {
            zero_acc();
            static_for<0, SPG, 1>([&](auto ssc) {
                constexpr int ss = decltype(ssc)::value;
                if (st + 1 < stage_end) prefetch(st + 1);
                const frag *tiles = reinterpret_cast<const frag *>(smem + (st & 1) * G.rec_bytes);
                mfma_run(tiles, std::integral_constant<int, STAGE_TILES>{},
                         std::integral_constant<int, ss * STAGE_TILES>{});
                if constexpr (ss == SPG - 1) epilogue(gr, nullptr);
                stage_sync();
                ++st;
            });
        }
    }

    // ---- outputs
    if (!SLICED && a.V_out) {
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
// The same sweep for wide games (N a multiple of 32 with two or four row tiles per type; leader
// rows in LDS; one type per stage).  Every wavefront sweeps TWO pairs of candidate tiles against
// each staged type, one pair after the other, so a workgroup of four wavefronts covers 512
// candidates per copy of the packed payoffs: stage copies (global memory -> LDS) slow the matrix
// pipe down roughly in proportion to the bytes a compute unit copies, and this halves them.  The
// fragments and the leader rows of a stage have LDS buffers of their own, two each; the one
// workgroup barrier per type stands at the start of the type, behind it the other buffers are free
// and the copies issued one type ago have landed, so a copy has a whole type to arrive.
// Epilogue: both candidate tiles of a pair advance together, stage by stage, so that every
// exchange with the partner lane (through the LDS crossbar) and every gather is in flight while
// the other tile's vector work is issued: per-tile lane maxima (which row tile holds the maximum)
// and element-wise maxima across the row tiles (which register position holds it); a unique
// maximiser is one tile and one position, anything else goes to the exact routine.  Arithmetic,
// operand order, packing and the exact-tie routine are those of sweep_mfma_kernel: the same bits
// per candidate.
template <typename T, int MP, int N, int WAVES, int PF>
__global__ void __launch_bounds__(WAVES * 64, 2)
sweep_wide_kernel(GameView g, SweepArgs a, int row_tiles)
{
    constexpr int NT = 2, NP = 2;              // candidate tiles per pass, passes per staged type
    typedef Path<T, MP> P;
    typedef typename P::frag frag;
    typedef typename P::xreg xreg;
    constexpr int KS = P::KSTEPS, HALF = P::HALF;
    constexpr Geometry G = make_geometry((int)sizeof(T), MP, N, N / 32, WAVES, true);
    constexpr int TPG = G.tpg;
    static_assert(N % 32 == 0 && (TPG == 2 || TPG == 4) && G.ts == 1, "one type of two or four row tiles per stage");
    static_assert(std::is_same<T, __bf16>::value, "bf16 matrix cores");
    constexpr int TILE_FRAGS = KS * 64;
    constexpr int FRAG_BYTES = TPG * G.tile_bytes;                      // the stage's fragments
    constexpr int LROW_CHUNKS = (G.at_bytes + 1023) / 1024;             // its leader rows, in 1 KiB copies
    constexpr int LROW_BYTES = LROW_CHUNKS * 1024;
    static_assert(FRAG_BYTES % (WAVES * 1024) == 0 && FRAG_BYTES + LROW_BYTES <= G.rec_bytes, "record layout");
    constexpr int NCH = TPG * KS / PF;                                  // fragment chunks per type
    static_assert(PF > 0 && KS % PF == 0 && NCH % 2 == 0, "chunk 0 of every pass lands in the same registers");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // F[2], then L[2]
    __shared__ float red_v[WAVES];
    __shared__ long long red_i[WAVES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, col = lane & 31;
    const int m = g.m, K = g.K;
    const unsigned char *records = reinterpret_cast<const unsigned char *>(g.Bpack);
    const unsigned char *ATpack = reinterpret_cast<const unsigned char *>(g.ATpack);
    const long long wave_base = ((long long)blockIdx.x * WAVES + wave) * (NP * NT * 32);
    const int partner_addr = 4 * (lane ^ 32);
    (void)row_tiles;

    auto copy_stage = [&](int st, int buf) __attribute__((always_inline)) {
        const unsigned char *src = records + (size_t)st * G.rec_bytes;
        unsigned char *dstF = smem + buf * FRAG_BYTES;
        unsigned char *dstL = smem + 2 * FRAG_BYTES + buf * LROW_BYTES;
#pragma unroll
        for (int i = 0; i < FRAG_BYTES / (WAVES * 1024); ++i) {
            const int chunk = i * WAVES + wave;
            __builtin_amdgcn_global_load_lds((global_ptr)(src + chunk * 1024 + lane * 16),
                                             (lds_ptr)(dstF + chunk * 1024), 16, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < (LROW_CHUNKS + WAVES - 1) / WAVES; ++i) {
            const int chunk = i * WAVES + wave;
            if (chunk < LROW_CHUNKS)                                     // wave-uniform
                __builtin_amdgcn_global_load_lds((global_ptr)(src + FRAG_BYTES + chunk * 1024 + lane * 16),
                                                 (lds_ptr)(dstL + chunk * 1024), 16, 0, 0);
        }
    };
    copy_stage(0, 0);

    // ---- candidate rows into registers (as in sweep_mfma_kernel), both passes
    constexpr int HALF_BASE = MP / 2;
    xreg x[NP][NT][P::XREGS];
    unsigned valid32[NP][NT];
#pragma unroll
    for (int ps = 0; ps < NP; ++ps)
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            const long long c = wave_base + (ps * NT + ct) * 32 + col;
            const bool ok = c < a.count;
            float vb[HALF_BASE];
            const float *row = a.X + (ok ? c : 0) * (long long)m + h * HALF_BASE;
            if (m == MP && HALF_BASE % 4 == 0 && ((uintptr_t)a.X & 15) == 0) {
#pragma unroll
                for (int e = 0; e < HALF_BASE; e += 4) {
                    f32x4 q = ok ? *(const f32x4 *)(row + e) : f32x4{ 0, 0, 0, 0 };
                    vb[e] = q[0]; vb[e + 1] = q[1]; vb[e + 2] = q[2]; vb[e + 3] = q[3];
                }
            } else {
#pragma unroll
                for (int e = 0; e < HALF_BASE; ++e) vb[e] = (ok && h * HALF_BASE + e < m) ? row[e] : 0.0f;
            }
            P::pack_x(vb, x[ps][ct]);
            valid32[ps][ct] = (unsigned)__builtin_amdgcn_ballot_w64(ok);
        }

    float V[NP][NT];
#pragma unroll
    for (int ps = 0; ps < NP; ++ps)
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) V[ps][ct] = 0.0f;
    unsigned tie_count = 0;                   // wave-uniform

    // Exact routine for one (candidate tile, type), as in sweep_mfma_kernel: the type's tiles once
    // more from the packed records in global memory (same instructions, same bits), the exact
    // maximisers in ascending action order, the leader's payoff decides and then the lower action.
    auto exact_type = [&](const xreg *xc, unsigned valid, int t, float gmax, float &l_out, int &j_out) __attribute__((always_inline)) {
        float lbest = 0.0f;
        int jbest = 0, nmatch = 0;
        const unsigned char *ATt = ATpack + (size_t)t * N * MP * sizeof(T);
#pragma unroll 1
        for (int tt = 0; tt < TPG; ++tt) {
            const frag *afrags = reinterpret_cast<const frag *>(
                records + (size_t)t * G.rec_bytes + (size_t)tt * G.tile_bytes);
            f32x16 acc1;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc1[r] = 0.0f;
#pragma unroll
            for (int s = 0; s < KS; ++s) acc1 = P::mfma(afrags[s * 64 + lane], xc, s, acc1);
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        const int r = 4 * q + rr;
                        const int j = tt * 32 + acc_row_base(r) + 4 * hh;
                        const unsigned long long meq = __builtin_amdgcn_ballot_w64(acc1[r] == gmax);
                        const unsigned hit = (unsigned)(hh ? (meq >> 32) : meq) & valid;
                        if (hit == 0u) continue;                       // wave-uniform
                        const float l = pair_sum(P::half_dot(xc, ATt + ((size_t)j * MP + h * HALF) * sizeof(T)));
                        if ((hit >> col) & 1u) {
                            if (nmatch == 0 || l > lbest) { lbest = l; jbest = j; }
                            ++nmatch;
                        }
                    }
        }
        l_out = lbest; j_out = jbest;
        tie_count += __builtin_popcount((unsigned)__builtin_amdgcn_ballot_w64(nmatch >= 2));
    };

    f32x16 acc[NT][TPG];
    frag fb[2][PF];
    auto read_chunk = [&](const frag *lane_base, auto qc, frag (&dst)[PF]) __attribute__((always_inline)) {
        constexpr int q = decltype(qc)::value;
#pragma unroll
        for (int e = 0; e < PF; ++e) {
            constexpr int f0 = q * PF;
            const int f = f0 + e;                                        // flat (tile, k-step)
            dst[e] = lane_base[(size_t)(f / KS) * TILE_FRAGS + (size_t)(f % KS) * 64];
        }
    };
    // MFMAs of one type for one pair of candidate tiles; chunk 0 of the fragments is already in
    // fb[0]; chunk q+1 is read before the MFMAs of chunk q are issued.
    auto mfma_type = [&](const frag *lane_base, const xreg (*xp)[P::XREGS]) __attribute__((always_inline)) {
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int tt = 0; tt < TPG; ++tt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[ct][tt][r] = 0.0f;
        static_for<0, NCH, 1>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            if constexpr (q + 1 < NCH) read_chunk(lane_base, std::integral_constant<int, q + 1>{}, fb[(q + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            static_for<0, PF, 1>([&](auto ec) {
                constexpr int f = q * PF + decltype(ec)::value;
                constexpr int tt = f / KS, ks = f % KS;
#pragma unroll
                for (int ct = 0; ct < NT; ++ct) acc[ct][tt] = P::mfma(fb[q & 1][decltype(ec)::value], xp[ct], ks, acc[ct][tt]);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    // Epilogue of type t for one pair of candidate tiles (rows xp, validity masks vp, values Vp);
    // leader rows of the type in Lt.
    auto epilogue = [&](int t, float pt, const lds_byte *Lt, const xreg (*xp)[P::XREGS], const unsigned *vp,
                        float *Vp, long long cbase) __attribute__((always_inline)) {
        // The asm blocks read the accumulators, and the compiler's hazard handling does not look into
        // inline asm: the wait states a vector read of a fresh MFMA result needs (passes + 3 = 11) are
        // explicit.
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_nop 15");
        // stage 1: per-tile lane maxima and element-wise maxima across the row tiles; the lane
        // maximum goes to the partner lane
        float pmt[NT][TPG], w[NT][16], pm[NT], pm_other[NT];
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            float u[TPG][16];
#pragma unroll
            for (int tt = 0; tt < TPG; ++tt)
#pragma unroll
                for (int r = 0; r < 16; ++r) u[tt][r] = acc[ct][tt][r];
            vmax16x2_first(pmt[ct][0], u[0], pmt[ct][TPG / 2], u[TPG / 2]);
            if constexpr (TPG == 4) {
                vmax16x2_first(pmt[ct][1], u[1], pmt[ct][3], u[3]);
                vmax4x16(w[ct], u[0], u[1], u[2], u[3]);
            } else {
                vmax2x16(w[ct], u[0], u[1]);
            }
            float p = TPG == 4 ? vmax3(pmt[ct][0], pmt[ct][1], pmt[ct][2]) : pmt[ct][0];
            pm[ct] = vmax2(p, pmt[ct][TPG - 1]);
            pm_other[ct] = pair_other(pm[ct], partner_addr);
            __builtin_amdgcn_sched_barrier(0);
        }
        // stage 2: the pair's maximum; the tile (exactly one per lane, or the columns are marked);
        // the position as a 16-bit map (bit 15 - r set iff position r holds the maximum); then
        // (action | number of maximisers << 16), zero in a lane without one, goes to the partner
        float gm[NT];
        unsigned total[NT], total_other[NT], tile_tie[NT];
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            gm[ct] = vmax2(pm[ct], pm_other[ct]);
            unsigned tile = 0u;
            unsigned long long seen = 0ull, dup = 0ull;
#pragma unroll
            for (int k = 0; k < TPG; ++k) {
                const bool e = pmt[ct][k] == gm[ct];
                const unsigned long long mk = __builtin_amdgcn_ballot_w64(e);
                dup |= seen & mk;
                seen |= mk;
                if (k) tile = e ? (unsigned)(32 * k) : tile;
            }
            tile_tie[ct] = (unsigned)(dup | (dup >> 32));
            const unsigned bm = bitmap16_pairs(w[ct], gm[ct]);
            const unsigned cnt = (unsigned)__builtin_popcount(bm);
            const unsigned r = ffbh(bm) - 16u;
            // action = 32 * tile + row(register) + 4h
            const unsigned act = tile | ((r & 0xCu) << 1) | (r & 3u) | (4u * h);
            total[ct] = cnt ? (cnt << 16) | act : 0u;
            total_other[ct] = (unsigned)__builtin_amdgcn_ds_bpermute(partner_addr, (int)total[ct]);
            __builtin_amdgcn_sched_barrier(0);
        }
        // stage 3: the action, the gather of its leader column, and whether the tile is clean
        int js[NT];
        bool clean[NT];
        typename P::colregs cr[NT];
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            const unsigned pair = total[ct] + total_other[ct];
            // (masked: a wavefront that is not clean may hold any sum here, and the gather is issued
            // before that is known)
            js[ct] = (int)(pair & 0xFFFFu);
            const unsigned jg = (N & (N - 1)) == 0 ? (unsigned)js[ct] & (unsigned)(N - 1)
                                                    : ((unsigned)js[ct] < (unsigned)N ? (unsigned)js[ct] : 0u);
            P::gather_half(Lt + (unsigned)((jg * G.ats + h * HALF) * sizeof(T)), cr[ct]);
            const unsigned multi = (unsigned)__builtin_amdgcn_ballot_w64((pair >> 16) != 1u) | tile_tie[ct];
            clean[ct] = (multi & vp[ct]) == 0u && vp[ct] == 0xFFFFFFFFu;   // wave-uniform
            __builtin_amdgcn_sched_barrier(0);
        }
        // stage 4: leader payoffs (each lane its half, the partner the other) and the value
        float l[NT];
        if (clean[0] && clean[1]) {
            float part[NT], part_other[NT];
            P::half_dot_regs2(xp[0], cr[0], xp[1], cr[1], part[0], part[1]);
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) part_other[ct] = pair_other(part[ct], partner_addr);
#pragma unroll
            for (int ct = 0; ct < NT; ++ct)
                l[ct] = h ? part_other[ct] + part[ct] : part[ct] + part_other[ct];      // (lower half) + (upper half)
        } else {
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) {
                if (clean[ct]) {
                    const float part = P::half_dot_regs(xp[ct], cr[ct]);
                    const float other = pair_other(part, partner_addr);
                    l[ct] = h ? other + part : part + other;
                } else {
                    exact_type(xp[ct], vp[ct], t, gm[ct], l[ct], js[ct]);
                }
            }
        }
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            Vp[ct] = fmaf(pt, l[ct], Vp[ct]);
            if (a.br_out) {
                const long long c = cbase + ct * 32 + col;
                if (h == 0 && c < a.count) a.br_out[c * K + t] = js[ct];
            }
        }
    };

    const frag *F0 = reinterpret_cast<const frag *>(smem) + lane;
    const frag *F1 = reinterpret_cast<const frag *>(smem + FRAG_BYTES) + lane;
    const lds_byte *L0 = (const lds_byte *)smem + (unsigned)(2 * FRAG_BYTES);
#pragma unroll 1
    for (int t = 0; t < K; ++t) {
        // own copies of this type's stage have landed; then everyone's have, and everyone is done with
        // the previous type, whose buffers take the next type's stage
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (t + 1 < K) copy_stage(t + 1, (t + 1) & 1);
        const float pt = g.prior[t];
        const frag *Ft = (t & 1) ? F1 : F0;
        const lds_byte *Lt = L0 + (unsigned)((t & 1) * LROW_BYTES);
        read_chunk(Ft, std::integral_constant<int, 0>{}, fb[0]);
#pragma unroll
        for (int ps = 0; ps < NP; ++ps) {
            mfma_type(Ft, x[ps]);
            if (ps + 1 < NP) read_chunk(Ft, std::integral_constant<int, 0>{}, fb[0]);   // the next pass's first fragments
            epilogue(t, pt, Lt, x[ps], valid32[ps], V[ps], wave_base + ps * NT * 32);
        }
    }

    // ---- outputs (as in sweep_mfma_kernel)
    if (a.V_out) {
#pragma unroll
        for (int ps = 0; ps < NP; ++ps)
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) {
                const long long c = wave_base + (ps * NT + ct) * 32 + col;
                float v = V[ps][ct];
                if (!(v == v)) v = -INFINITY;
                if (h == 0 && c < a.count) a.V_out[c] = v;
            }
    }
    if (a.blk_v) {
        float bv = -INFINITY;
        long long bi = LLONG_MAX;
#pragma unroll
        for (int ps = 0; ps < NP; ++ps)
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) {
                const long long c = wave_base + (ps * NT + ct) * 32 + col;
                float v = V[ps][ct];
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
            for (int w2 = 1; w2 < WAVES; ++w2)
                if (red_v[w2] > bv || (red_v[w2] == bv && red_i[w2] < bi)) { bv = red_v[w2]; bi = red_i[w2]; }
            a.blk_v[blockIdx.x] = bv;
            a.blk_i[blockIdx.x] = bi;
        }
    }
    if (a.tie_counter && lane == 0 && tie_count) atomicAdd(a.tie_counter, (unsigned long long)tie_count);
}

// Second step of the type-sliced evaluation: V[c] = sum_t prior[t] * l[c][t], one lane per row,
// accumulated in type order with the fused multiply-add of the unsliced kernel, so the value is
// the same fp32 number.
__global__ void finish_value_kernel(const float *__restrict__ prior, const float *__restrict__ l,
                                    int K, long long count, float *__restrict__ V_out)
{
    const long long c = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= count) return;
    float v = 0.0f;
    for (int t = 0; t < K; ++t) v = fmaf(prior[t], l[c * K + t], v);
    if (!(v == v)) v = -INFINITY;
    V_out[c] = v;
}

// ------------------------------------------------------------------------------------------
// Instantiation table.
struct Variant {
    int mode;                    // 0 fp32 MFMA, 1 bf16 MFMA on rounded operands, 2 bf16 MFMA on split fp32
    int terms;                   // 1, or the number of part products of the split (3 or 6)
    int mp_base, n, nt, waves, stage_tiles;
    bool at_lds;
    void (*kernel)(GameView, SweepArgs, int);     // null when `wide` sweeps this packing
    void (*sliced)(GameView, SweepArgs, int);     // one candidate tile per wavefront, types sliced
    Geometry geo;
    const char *name;
    void (*wide)(GameView, SweepArgs, int);       // sweep_wide_kernel for this packing, or null
    int wide_lds;                                 // its dynamic LDS bytes
};

#define BSSE_VARIANT(T, MODE, TERMSv, MPB, Nv, NTv, Wv, STv, OCCv, ATL, PFv, NAME)                   \
    { MODE, TERMSv, MPB, Nv, NTv, Wv, STv, ATL,                                                      \
      sweep_mfma_kernel<T, MPB * TERMSv, Nv, NTv, Wv, STv, OCCv, ATL, TERMSv, false, PFv>,           \
      sweep_mfma_kernel<T, MPB * TERMSv, Nv, 1, Wv, STv, 1, ATL, TERMSv, true, PFv>,                 \
      make_geometry((int)sizeof(T), MPB * TERMSv, Nv, STv, Wv, ATL, TERMSv), NAME, nullptr, 0 }
// A packing that sweep_wide_kernel also takes (one type per stage, leader rows in LDS, NT = 2)
#define BSSE_VARIANT_WIDE(T, MODE, MPB, Nv, Wv, PFv, NAME)                                           \
    { MODE, 1, MPB, Nv, 2, Wv, Nv / 32, true,                                                        \
      nullptr,                                                                                       \
      sweep_mfma_kernel<T, MPB, Nv, 1, Wv, Nv / 32, 1, true, 1, true, PFv>,                          \
      make_geometry((int)sizeof(T), MPB, Nv, Nv / 32, Wv, true), NAME,                               \
      sweep_wide_kernel<T, MPB, Nv, Wv, PFv>, wide_lds_bytes((int)sizeof(T), MPB, Nv, Wv) }

const Variant kVariants[] = {
    // fp32 MFMA (the last number before the name: k-steps per fragment read-ahead chunk, 0 = the
    // fragment reads are left where they are used)
    BSSE_VARIANT(float, 0, 1, 8, 8, 4, 4, 1, 2, true, 0, "mfma_f32"),
    BSSE_VARIANT(float, 0, 1, 16, 16, 4, 4, 2, 2, true, 0, "mfma_f32"),
    BSSE_VARIANT(float, 0, 1, 32, 32, 4, 4, 4, 2, true, 0, "mfma_f32"),
    BSSE_VARIANT(float, 0, 1, 32, 64, 2, 4, 4, 2, true, 0, "mfma_f32"),
    BSSE_VARIANT(float, 0, 1, 128, 256, 1, 4, 2, 2, false, 0, "mfma_f32"),
    // bf16 MFMA, operands rounded to bf16
    BSSE_VARIANT(__bf16, 1, 1, 16, 32, 4, 4, 2, 2, true, 0, "mfma_bf16"),
    BSSE_VARIANT(__bf16, 1, 1, 32, 16, 4, 4, 2, 2, false, 0, "mfma_bf16"),
    BSSE_VARIANT_WIDE(__bf16, 1, 64, 128, 8, 4, "mfma_bf16"),
    // bf16 MFMA on fp32 operands split into bf16 parts
    BSSE_VARIANT(__bf16, 2, 6, 16, 16, 2, 4, 2, 2, true, 0, "mfma_split6"),
    BSSE_VARIANT(__bf16, 2, 6, 32, 32, 2, 4, 1, 3, true, 0, "mfma_split6"),
    BSSE_VARIANT(__bf16, 2, 3, 32, 32, 4, 4, 4, 2, true, 0, "mfma_split3"),
    BSSE_VARIANT(__bf16, 2, 6, 32, 64, 2, 4, 2, 2, true, 0, "mfma_split6"),
    BSSE_VARIANT(__bf16, 2, 3, 128, 256, 1, 8, 8, 2, false, 0, "mfma_split3"),
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));
constexpr int kSmallVariant = 1000;          // the small-game kernel (sweep_small.hip)

int row_tiles_for(const Variant &v, int K)
{
    if (v.n >= 32) return K * (v.n / 32);
    const int tpt = 32 / v.n;
    return (K + tpt - 1) / tpt;
}

// bf16 parts of a value: hi, mid, lo with v = hi + mid + lo up to the rounding of lo
void bf16_parts(float v, float part[3])
{
    auto rne = [](float f) {
        uint32_t b; memcpy(&b, &f, 4);
        b += 0x7FFFu + ((b >> 16) & 1u);
        b &= 0xFFFF0000u;
        memcpy(&f, &b, 4);
        return f;
    };
    part[0] = rne(v);
    const float r1 = v - part[0];
    part[1] = rne(r1);
    const float r2 = r1 - part[1];
    part[2] = rne(r2);
}

}  // namespace

int mfma_select(int m, int n, int K, int mode, bool exact)
{
    if (mode == 0 && small_supported(m, n, K, 0)) return kSmallVariant;
    int best = -1;
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant &v = kVariants[i];
        if (v.mode != mode || v.n != n || v.mp_base < m) continue;
        if (v.terms == 3 && !exact) continue;
        // smallest padded m wins; among equals, fewer terms
        if (best < 0 || v.mp_base < kVariants[best].mp_base ||
            (v.mp_base == kVariants[best].mp_base && v.terms < kVariants[best].terms))
            best = i;
    }
    return best;
}

const char *mfma_variant_name(int variant)
{
    if (variant == kSmallVariant) return "mfma_small_split6";
    return (variant >= 0 && variant < kNumVariants) ? kVariants[variant].name : "";
}

bool mfma_is_small(int variant) { return variant == kSmallVariant; }
bool mfma_slices_types(int variant) { return variant >= 0 && variant < kNumVariants; }

long long mfma_num_blocks(int variant, long long count)
{
    if (variant == kSmallVariant) return small_num_blocks(count);
    const Variant &v = kVariants[variant];
    const long long per = (long long)v.nt * 32 * v.waves * (v.wide ? 2 : 1);     // candidates per workgroup record     // candidates per workgroup record
    return (count + per - 1) / per;
}

// Once per game, on the game's device: kernels whose two stage buffers exceed the default 48 KiB of
// dynamic LDS get their limit raised here, not at every launch.
hipError_t mfma_prepare(int variant, int K)
{
    if (variant == kSmallVariant) return hipSuccess;
    if (variant < 0 || variant >= kNumVariants) return hipErrorNotSupported;
    const Variant *v = &kVariants[variant];
    const int tiles = row_tiles_for(*v, K);
    const int nstages = (tiles + v->stage_tiles - 1) / v->stage_tiles;
    const size_t lds = (size_t)v->geo.rec_bytes * (nstages > 1 ? 2 : 1);
    if (v->wide && v->wide_lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)v->wide, hipFuncAttributeMaxDynamicSharedMemorySize, v->wide_lds);
        if (e != hipSuccess) return e;
    }
    if (lds <= 48 * 1024) return hipSuccess;
    hipError_t e = hipSuccess;
    if (v->kernel) e = hipFuncSetAttribute((const void *)v->kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void *)v->sliced, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    return e;
}

hipError_t launch_sweep_mfma(const GameView &g, const SweepArgs &a, hipStream_t s)
{
    if (a.count <= 0) return hipSuccess;
    if (g.variant == kSmallVariant) return launch_sweep_small(g, a, s);
    if (g.variant < 0 || g.variant >= kNumVariants) return hipErrorNotSupported;
    const Variant *v = &kVariants[g.variant];
    const int tiles = row_tiles_for(*v, g.K);
    const int nstages = (tiles + v->stage_tiles - 1) / v->stage_tiles;
    const size_t lds = (size_t)v->geo.rec_bytes * (nstages > 1 ? 2 : 1);
    auto kernel = a.l_out ? v->sliced : v->kernel;     // (mfma_prepare has raised their LDS limit)
    if (!a.l_out) {
        const long long blocks = mfma_num_blocks(g.variant, a.count);
        if (v->wide)       // (every wavefront sweeps two pairs of candidate tiles)
            hipLaunchKernelGGL(v->wide, dim3((unsigned)blocks), dim3(v->waves * 64), (size_t)v->wide_lds, s, g, a, tiles);
        else
            hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(v->waves * 64), lds, s, g, a, tiles);
        return hipGetLastError();
    }
    // type-sliced evaluation: 32 candidates per wavefront, whole groups per slice; few rows are
    // cut into about 256 slices, many rows fill the chip by themselves
    const long long per = 32LL * v->waves, blocks = (a.count + per - 1) / per;
    if (a.blk_v || blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    const int kSlices = blocks >= 256 ? 1 : (int)(256 / blocks);
    const int spg = v->geo.tpg > v->stage_tiles ? v->geo.tpg / v->stage_tiles : 1;   // stages per group
    SweepArgs b = a;
    b.slice_stages = ((nstages + kSlices - 1) / kSlices + spg - 1) / spg * spg;
    const int slices = (nstages + b.slice_stages - 1) / b.slice_stages;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks, (unsigned)slices), dim3(v->waves * 64), lds, s, g, b,
                       tiles);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !a.V_out) return e;
    hipLaunchKernelGGL(finish_value_kernel, dim3((unsigned)((a.count + 63) / 64)), dim3(64), 0, s,
                       g.prior, a.l_out, g.K, a.count, a.V_out);
    return hipGetLastError();
}

// Host packing.
// The contraction index of a variant runs over MP = terms * mp_base slots.  Lane half h owns
// slots h*MP/2 .. (h+1)*MP/2; within a half, slot = term * mp_base/2 + (i - h*mp_base/2) for the
// leader actions i of that half, and the value stored at (term, i) is part q(term) of the payoff:
// the payoff itself when terms == 1, parts (0,1,0,2,1,0) for six terms, (0,0,0) for three (whose
// fragments hold the first block only: the kernel uses each for all three terms).
// Bpack = stage records (see Geometry): per stage, STAGE_TILES row tiles, each laid out as
// [k-step][lane 0..63][fragment], where lane = 32*h + rowInTile supplies the slots
// h*MP/2 + (elements per lane)*s + e of (type, action) row 32*tile + rowInTile; then, when the
// variant keeps leader rows in LDS, the rows [type slot][action][MP + pad] of the types the
// stage covers, in the same slot order.  Rows past K*n and actions past m are zero.
// ATpack = [K][n][MP] leader payoffs in slot order (zero padded), so that a lane's half of a
// column is contiguous; used by the global gather and by the exact routine.  Six-term variants that
// keep leader rows in LDS carry them as plain fp32 instead, in the stage records ([type slot]
// [action][mp_base + 4]) and in ATpack ([K][n][mp_base]).
void mfma_pack(int variant, int m, int n, int K, const float *A, const float *B, void **Bpack,
               size_t *Bbytes, void **ATpack, size_t *ATbytes, int *m_pad, int *n_pad)
{
    *Bpack = nullptr; *ATpack = nullptr; *Bbytes = 0; *ATbytes = 0;
    if (variant == kSmallVariant) {
        *m_pad = 8; *n_pad = n;
        small_pack(m, n, K, A, B, Bpack, Bbytes, ATpack, ATbytes);
        return;
    }
    if (variant < 0 || variant >= kNumVariants) return;
    const Variant *v = &kVariants[variant];
    const Geometry &G = v->geo;
    const int MP = v->mp_base * v->terms, half = MP / 2, half_base = v->mp_base / 2;
    const bool bf = v->mode != 0;
    const int epl = bf ? 8 : 1;                            // k-slots per lane per MFMA
    const int ks = half / epl / (v->terms == 3 ? 3 : 1);   // fragment k-steps per tile (one block of three-term rows)
    const int tiles = row_tiles_for(*v, K);
    const int nstages = (tiles + v->stage_tiles - 1) / v->stage_tiles;
    const size_t esz = bf ? 2 : 4;
    static const int bsel6[6] = { 0, 1, 0, 2, 1, 0 };
    *m_pad = v->mp_base; *n_pad = n;
    *Bbytes = (size_t)nstages * G.rec_bytes;
    const bool lead_f32 = v->terms == 6 && v->at_lds;       // leader rows as plain fp32
    *ATbytes = lead_f32 ? (size_t)K * n * v->mp_base * sizeof(float) : (size_t)K * n * MP * esz;
    unsigned char *pb = (unsigned char *)calloc(*Bbytes, 1);
    unsigned char *pa = (unsigned char *)calloc(*ATbytes, 1);
    if (!pb || !pa) { free(pb); free(pa); return; }
    auto put = [&](unsigned char *base, size_t idx, float val) {
        if (bf) {
            uint32_t b; memcpy(&b, &val, 4);
            b += 0x7FFFu + ((b >> 16) & 1u);
            const uint16_t hb = (uint16_t)(b >> 16);
            memcpy(base + idx * 2, &hb, 2);
        } else {
            memcpy(base + idx * 4, &val, 4);
        }
    };
    // value stored at slot `li` (within lane half hh) of payoff matrix M (type t, action j)
    auto slot_value = [&](const float *M, int t, int j, int hh, int li) -> float {
        const int term = li / half_base, i = hh * half_base + li % half_base;
        if (t >= K || i >= m) return 0.0f;
        const float val = M[((size_t)t * m + i) * n + j];
        if (v->terms == 1) return val;
        float part[3];
        bf16_parts(val, part);
        return part[v->terms == 3 ? 0 : bsel6[term]];
    };
    for (int tile = 0; tile < tiles; ++tile) {
        unsigned char *tb = pb + (size_t)(tile / v->stage_tiles) * G.rec_bytes +
                            (size_t)(tile % v->stage_tiles) * G.tile_bytes;
        for (int s = 0; s < ks; ++s)
            for (int lane = 0; lane < 64; ++lane) {
                const int hh = lane / 32, row = tile * 32 + lane % 32;
                const int t = row / n, j = row % n;
                for (int e = 0; e < epl; ++e)
                    put(tb, ((size_t)s * 64 + lane) * epl + e, slot_value(B, t, j, hh, epl * s + e));
            }
    }
    if (v->at_lds)
        for (int st = 0; st < nstages; ++st) {
            unsigned char *ab = pb + (size_t)st * G.rec_bytes + (size_t)v->stage_tiles * G.tile_bytes;
            for (int q = 0; q < G.ts; ++q) {
                const int t = st * G.ts + q;
                if (t >= K) break;
                for (int j = 0; j < n; ++j) {
                    if (lead_f32) {
                        float *row = reinterpret_cast<float *>(ab + ((size_t)q * n + j) * G.ats * esz);
                        for (int i = 0; i < v->mp_base; ++i) row[i] = i < m ? A[((size_t)t * m + i) * n + j] : 0.0f;
                        continue;
                    }
                    for (int hh = 0; hh < 2; ++hh)
                        for (int li = 0; li < half; ++li)
                            put(ab, ((size_t)q * n + j) * G.ats + hh * half + li, slot_value(A, t, j, hh, li));
                }
            }
        }
    for (int t = 0; t < K; ++t)
        for (int j = 0; j < n; ++j) {
            if (lead_f32) {
                float *row = reinterpret_cast<float *>(pa) + ((size_t)t * n + j) * v->mp_base;
                for (int i = 0; i < v->mp_base; ++i) row[i] = i < m ? A[((size_t)t * m + i) * n + j] : 0.0f;
                continue;
            }
            for (int hh = 0; hh < 2; ++hh)
                for (int li = 0; li < half; ++li)
                    put(pa, ((size_t)t * n + j) * MP + hh * half + li, slot_value(A, t, j, hh, li));
        }
    *Bpack = pb; *ATpack = pa;
}

}  // namespace bsse
