// Guard-free grouped GEMM over bf16 terms on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// Operands.  A real matrix enters the product as NT bf16 terms whose sum approximates it: term 0
// is the value rounded to bf16, term 1 the rounded remainder (8 / 16 significant bits for NT = 1 /
// 2).  An operand is either a plain bf16 matrix (NT = 1), a plain fp32 matrix that the loader cuts
// into two terms while it stages it (FA / FB), or a matrix stored as terms: interleaved along k in
// groups of 32, a row holds, for every 32 consecutive k, NT segments of 32 bf16 (64 bytes) - term
// 0's values, then term 1's - so that element (r, k) of term t sits at
// r * ld + (k / 32) * (32 NT) + t * 32 + k % 32 and, with NT = 2, one k-group of a row is one
// 128-byte cache line (row pieces of 64 bytes run at half the load bandwidth: 17 against 34 TB/s
// from L2).  The LDS layout is that of the stored terms in every case.  A product of two operands
// is the sum of the term-pair products selected by a compile-time mask; every pair is an exact
// bf16 x bf16 product accumulated in fp32.
//
// One launch walks a device table of problems  C = alpha A B^T + beta C  (A is M x K, B is
// N x K, both k-contiguous).  Symmetric problems compute the tiles on or below the diagonal and
// mirror them.  Operand rows are whole tiles and K whole slabs (the callers send other shapes to
// the guarded kernels), so the K loop has no guards; the fp32 output is guarded.
#pragma once
#include <type_traits>

#include "gemm.h"

namespace asteria {

typedef __bf16 pg_bf16x8 __attribute__((ext_vector_type(8)));

constexpr int PG_GROUP = 32;   // k values per interleave group

struct PlaneProblem {
    const void *A;          // split / bf16 matrix (NTA terms), or fp32 matrix when the shape says so
    const void *B;          // the same for B
    float *C32;             // fp32 output
    int M, N, K;
    int lda, ldb, ldc32;    // elements
    int tile_start;
    int tiles_n;            // tile columns (non-symmetric problems)
    int state_idx, state_mask;
    float alpha, beta;
    int flags;              // GEMM_SYM, GEMM_C_PACKED, GEMM_STORE_T (output stored transposed, no beta), PG_KMAJOR
};

// pair (ta, tb) of an NTA x NTB split product is issued iff bit ta * 2 + tb of PAIRS is set
// problem flag (beside the GEMM_* ones): both operands are plain bf16 matrices stored k-major
constexpr int PG_KMAJOR = 16;

constexpr unsigned PG_PAIRS_1 = 0x1u;            // (0,0)
constexpr unsigned PG_PAIRS_2x1 = 0x1u | 0x4u;   // (0,0) (1,0)
constexpr unsigned PG_PAIRS_1x2 = 0x1u | 0x2u;   // (0,0) (0,1)
constexpr unsigned PG_PAIRS_2x2 = 0x7u;          // (0,0) (0,1) (1,0): 16 bits of both operands

// WGM x WGN wavefronts of WTM x WTN MFMA tiles (32 x 32); K slabs of BK; DEPTH register sets
// of global-load prefetch.
template <int NTA_, int NTB_, unsigned PAIRS_, int WGM_, int WGN_, int WTM_, int WTN_, int BK_, int DEPTH_ = 1, int MODE_ = 0,
          bool FA_ = false, bool FB_ = false, bool KM_ = false>
struct PgShape {
    // KM: the kernel also accepts problems flagged PG_KMAJOR, whose operands are bf16 matrices stored
    // k-major (A'(i, k) = A[k * lda + i]); one term, 128 x 128 tiles of 4 wavefronts, slabs of 64
    static constexpr bool KM = KM_;
    static_assert(!KM_ || (NTA_ == 1 && NTB_ == 1 && WGM_ == 2 && WGN_ == 2 && WTM_ == 2 && WTN_ == 2 && BK_ == 64 &&
                           !FA_ && !FB_ && MODE_ == 0),
                  "k-major problems: plain bf16, 128 x 128 tiles, slabs of 64");
    // FA / FB: the operand is a plain fp32 row-major matrix, split into two bf16 terms while it is
    // staged (the LDS layout is that of a two-term split matrix); it then needs NT = 2
    static constexpr bool FA = FA_, FB = FB_;
    static_assert((!FA_ || NTA_ == 2) && (!FB_ || NTB_ == 2), "fp32 sources are split into two terms");
    static constexpr int NTA = NTA_, NTB = NTB_, DEPTH = DEPTH_;
    static constexpr int MODE = MODE_;                   // 0: every wavefront loads and multiplies in turn; 1: two wavefront groups alternate
    static constexpr unsigned PAIRS = PAIRS_;
    static constexpr int WGM = WGM_, WGN = WGN_, WTM = WTM_, WTN = WTN_, BK = BK_;
    static constexpr int TM = 32 * WTM * WGM, TN = 32 * WTN * WGN;   // workgroup tile
    static constexpr int NTHR = 64 * WGM * WGN;
    static constexpr int GPS = BK / PG_GROUP;            // interleave groups per slab
    static constexpr int CPG = PG_GROUP / 8;             // 16-byte chunks per term segment (4)
    // an LDS row of an operand holds the slab piece of one matrix row as it lies in memory:
    // GPS groups x NT segments x 4 chunks; chunks are XOR-swizzled by row
    static constexpr int CPR_A = GPS * NTA * CPG, CPR_B = GPS * NTB * CPG;
    static constexpr int RPV_A = NTHR / CPR_A, RPV_B = NTHR / CPR_B;   // rows covered by one vector index
    static constexpr int NVA = TM / RPV_A, NVB = TN / RPV_B;
    static constexpr int ROW_A = CPR_A * 8, ROW_B = CPR_B * 8;         // elements per LDS row
    static constexpr int STAGE = TM * ROW_A + TN * ROW_B;              // elements per stage
    static constexpr int STEPS = BK / 16;                // MFMA k-steps per slab
    static constexpr size_t LDS_MAIN = 2 * (size_t)STAGE * sizeof(uint16_t);
    static constexpr int CT_PITCH = 136;                 // fp32 staging tile of the epilogue (128 x 128)
    static constexpr size_t LDS_EPI = 128 * (size_t)CT_PITCH * sizeof(float);
    static constexpr size_t LDS_BYTES = LDS_MAIN > LDS_EPI ? LDS_MAIN : LDS_EPI;
    static_assert(BK % PG_GROUP == 0, "slab = whole interleave groups");
    static_assert(TM % 128 == 0 && TN % 128 == 0 && TM == TN, "square tiles of 128 x 128 quadrants");
    static_assert(NTHR % CPR_A == 0 && NTHR % CPR_B == 0 && TM % RPV_A == 0 && TN % RPV_B == 0, "loader geometry");
    static_assert((CPR_A & (CPR_A - 1)) == 0 && (CPR_B & (CPR_B - 1)) == 0 && CPR_A <= 16 && CPR_B <= 16 &&
                      RPV_A % 16 == 0 && RPV_B % 16 == 0, "swizzle geometry");
    static_assert(NTA >= 1 && NTA <= 2 && NTB >= 1 && NTB <= 2, "one or two terms");
};

// chunk c of LDS row r (CPR chunks per row) is stored at position c ^ swz(r): a 16-lane group
// of the loader then writes whole contiguous rows, and the 16 rows a lane group reads for one
// fragment chunk fall into 16 distinct 16-byte bank groups
template <int CPR> __device__ __forceinline__ int pg_swz(int r) { return (r / (16 / CPR)) % CPR; }

__device__ __forceinline__ floatx16 pg_mma(u32x4 a, u32x4 b, floatx16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(pg_bf16x8, a), __builtin_bit_cast(pg_bf16x8, b),
                                                   c, 0, 0, 0);
}

// LDS-only barrier: waits for this wavefront's LDS traffic, not for its global loads in flight
__device__ __forceinline__ void pg_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ uint32_t pg_pack_bf16(float a, float b)
{
    const __bf16 x = (__bf16)a, y = (__bf16)b;   // v_cvt_pk_bf16_f32: round to nearest even
    return (uint32_t)__builtin_bit_cast(uint16_t, x) | ((uint32_t)__builtin_bit_cast(uint16_t, y) << 16);
}

// Global -> register -> LDS staging of one operand's slab pieces.  Pre-split / bf16 source: one
// 16-byte chunk per item, stored as loaded.  fp32 source: an item is 8 consecutive fp32 (two
// 16-byte loads) and becomes one hi chunk and one lo chunk (round to nearest in both terms).
template <class S, bool F32, int NT, int TROWS>
struct PgLoader {
    static constexpr int CPR = S::GPS * NT * S::CPG;      // 16-byte chunks per LDS row
    static constexpr int ROW = CPR * 8;                    // elements per LDS row
    static constexpr int IPR = F32 ? S::BK / 8 : CPR;      // items per row
    static constexpr int RPV = S::NTHR / IPR;              // rows covered by one item index
    static constexpr int NV = TROWS / RPV;
    static constexpr int RPI = F32 ? 2 : 1;                // 16-byte registers per item
    static constexpr int SRC_BYTES = F32 ? 4 : 2;
    static constexpr int SLAB_BYTES = F32 ? S::BK * 4 : S::BK * NT * 2;   // bytes of one slab piece of a row
    static_assert(S::NTHR % IPR == 0 && TROWS % RPV == 0 && RPV % 16 == 0, "loader geometry");
    u32x4 r[S::DEPTH][NV][RPI];
    const char *ub;      // wave-uniform base: the loads need no 64-bit vector address arithmetic
    uint32_t vo;         // per-thread byte offset
    size_t step;         // bytes between the rows of consecutive item indices
    uint32_t lds_hi, lds_lo;   // element offsets of this thread's chunk(s) inside the operand's LDS block

    __device__ __forceinline__ void init(const void *base, int ld, int row0, int tid)
    {
        const int lrow = tid / IPR, item = tid % IPR;
        ub = reinterpret_cast<const char *>(base) + (size_t)row0 * ld * SRC_BYTES;
        vo = ((uint32_t)lrow * (uint32_t)ld + (uint32_t)item * 8u) * SRC_BYTES;
        step = (size_t)RPV * ld * SRC_BYTES;
        const int sw = pg_swz<CPR>(lrow);
        if (F32) {
            const int g = item / S::CPG, q = item % S::CPG;          // interleave group, chunk inside a term segment
            lds_hi = (uint32_t)(lrow * ROW + (((g * 2) * S::CPG + q) ^ sw) * 8);
            lds_lo = (uint32_t)(lrow * ROW + (((g * 2 + 1) * S::CPG + q) ^ sw) * 8);
        } else {
            lds_hi = (uint32_t)(lrow * ROW + ((item ^ sw) * 8));
            lds_lo = 0;
        }
    }
    template <int SET> __device__ __forceinline__ void gload(int slab)
    {
        const size_t k = (size_t)slab * SLAB_BYTES;
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int e = 0; e < RPI; ++e)
                r[SET][v][e] = *(const ASTERIA_GLOBAL u32x4 *)(ub + (v * step + k + 16 * e) + vo);
    }
    template <int SET> __device__ __forceinline__ void lstore(ASTERIA_LDS uint16_t *d) const
    {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            if constexpr (F32) {
                u32x4 hi, lo;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const u32x4 x = r[SET][v][e];
                    const float x0 = __uint_as_float(x[0]), x1 = __uint_as_float(x[1]);
                    const float x2 = __uint_as_float(x[2]), x3 = __uint_as_float(x[3]);
                    const uint32_t h0 = pg_pack_bf16(x0, x1), h1 = pg_pack_bf16(x2, x3);
                    hi[2 * e] = h0; hi[2 * e + 1] = h1;
                    lo[2 * e] = pg_pack_bf16(x0 - __uint_as_float(h0 << 16), x1 - __uint_as_float(h0 & 0xffff0000u));
                    lo[2 * e + 1] = pg_pack_bf16(x2 - __uint_as_float(h1 << 16), x3 - __uint_as_float(h1 & 0xffff0000u));
                }
                *(ASTERIA_LDS u32x4 *)(d + lds_hi + v * RPV * ROW) = hi;
                *(ASTERIA_LDS u32x4 *)(d + lds_lo + v * RPV * ROW) = lo;
            } else {
                *(ASTERIA_LDS u32x4 *)(d + lds_hi + v * RPV * ROW) = r[SET][v][0];
            }
        }
    }
};


// One finished row piece of 8 values at (grow, gcol .. gcol + 7): apply beta, store.
// `ctile`: for packed lower-tile output the base of the 128 x 128 tile this piece belongs to (row lr of
// it, 128 floats per row), else null (row-major output at C32 + grow ldc32).
__device__ __forceinline__ void pg_emit(const PlaneProblem &P, int grow, int gcol, int rlim, int clim, float (&val)[8],
                                        float *ctile = nullptr)
{
    if (grow >= rlim) return;
    float *c = ctile ? ctile + (size_t)(grow % PACK_T) * PACK_T + (gcol % PACK_T) : P.C32 + (size_t)grow * P.ldc32 + gcol;
    const bool vec = (gcol + 8 <= clim) && (ctile || (P.ldc32 & 3) == 0) && ((reinterpret_cast<uintptr_t>(P.C32) & 15u) == 0);
    if (vec) {
        ASTERIA_GLOBAL floatx4 *c4 = (ASTERIA_GLOBAL floatx4 *)c;
        if (P.beta != 0.0f) {
            const floatx4 o0 = c4[0], o1 = c4[1];
#pragma unroll
            for (int e = 0; e < 4; ++e) { val[e] += P.beta * o0[e]; val[4 + e] += P.beta * o1[e]; }
        }
        floatx4 s0, s1;
#pragma unroll
        for (int e = 0; e < 4; ++e) { s0[e] = val[e]; s1[e] = val[4 + e]; }
        c4[0] = s0; c4[1] = s1;
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (gcol + e < clim) {
                if (P.beta != 0.0f) val[e] += P.beta * c[e];
                c[e] = val[e];
            }
    }
}

// K loop of a 128 x 128 tile whose operands lie k-major in memory (G^T G read from G as it is).
// A slab is 64 rows (k) of 128 consecutive elements per operand and is staged as it lies in memory:
// LDS row = k, 256 bytes, its four 64-byte segments XOR-swizzled by k % 4.  The MFMA operands (8
// consecutive k of one row i per lane) come out of LDS through ds_read_b64_tr_b16, which transposes
// within 16 lanes: lane 4 e + q supplies the address of elements 4 q .. 4 q + 3 of row k0 + e, and
// lane j receives element j of rows k0 .. k0 + 3.  Two such reads give the 8 values of a lane; a
// 32-lane half then touches 4 rows x 64 bytes, which the swizzle spreads over all 64 banks.
template <class S>
__device__ __forceinline__ void pg_kmajor_loop(floatx16 (&acc)[2][2], const PlaneProblem &P, int row0, int col0,
                                               ASTERIA_LDS uint16_t *smem, int tid, int wm, int wn, int lane)
{
    constexpr int BK = 64, ROWB = 256, OPB = BK * ROWB, STAGEB = 2 * OPB;
    static_assert(2 * STAGEB <= (int)S::LDS_BYTES, "two stages fit");
    typedef short pg_short4 __attribute__((ext_vector_type(4)));
    ASTERIA_LDS char *lds = (ASTERIA_LDS char *)smem;
    // loader: thread -> 16-byte vector v of slab row kr (+ 16 per register)
    const int v = tid & 15, kr = tid >> 4;
    const char *ga = reinterpret_cast<const char *>(P.A) + ((size_t)row0 + 8 * v) * 2 + (size_t)kr * P.lda * 2;
    const char *gb = reinterpret_cast<const char *>(P.B) + ((size_t)col0 + 8 * v) * 2 + (size_t)kr * P.ldb * 2;
    const size_t stepa = (size_t)16 * P.lda * 2, stepb = (size_t)16 * P.ldb * 2;       // 16 rows on
    const size_t slaba = (size_t)BK * P.lda * 2, slabb = (size_t)BK * P.ldb * 2;
    // (kr + 16 vi) % 4 = kr % 4: one store offset serves the four registers
    const uint32_t st_off = (uint32_t)(kr * ROWB + (((v >> 2) ^ (kr & 3)) << 6) + ((v & 3) << 4));
    u32x4 ra[4], rb[4];
    auto gload = [&](int slab) {
#pragma unroll
        for (int vi = 0; vi < 4; ++vi) {
            ra[vi] = *(const ASTERIA_GLOBAL u32x4 *)(ga + slab * slaba + vi * stepa);
            rb[vi] = *(const ASTERIA_GLOBAL u32x4 *)(gb + slab * slabb + vi * stepb);
        }
    };
    auto lstore = [&](int stage) {
#pragma unroll
        for (int vi = 0; vi < 4; ++vi) {
            *(ASTERIA_LDS u32x4 *)(lds + stage * STAGEB + st_off + vi * 16 * ROWB) = ra[vi];
            *(ASTERIA_LDS u32x4 *)(lds + stage * STAGEB + OPB + st_off + vi * 16 * ROWB) = rb[vi];
        }
    };
    // fragment reads: 16-lane group g = (k half, i half), lane 4 e + q of it reads row e, elements 4 q ..
    const int g = lane >> 4, e = (lane >> 2) & 3, q = lane & 3;
    const uint32_t rd_row = (uint32_t)((8 * (g >> 1) + e) * ROWB);
    const uint32_t rd_col = (uint32_t)((16 * (g & 1) + 4 * q) * 2);
    uint32_t fa[2], fb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        fa[i] = rd_row + ((uint32_t)((wm * 2 + i) ^ e) << 6) + rd_col;
        fb[i] = (uint32_t)OPB + rd_row + ((uint32_t)((wn * 2 + i) ^ e) << 6) + rd_col;
    }
    auto frag = [&](uint32_t off) {
        const pg_short4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ASTERIA_LDS pg_short4 *)(lds + off));
        const pg_short4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ASTERIA_LDS pg_short4 *)(lds + off + 4 * ROWB));
        typedef uint32_t pg_u32x2 __attribute__((ext_vector_type(2)));
        const pg_u32x2 l2 = __builtin_bit_cast(pg_u32x2, lo), h2 = __builtin_bit_cast(pg_u32x2, hi);
        u32x4 r;
        r[0] = l2[0]; r[1] = l2[1]; r[2] = h2[0]; r[3] = h2[1];
        return r;
    };
    const int nk = P.K / BK;
    gload(0);
    lstore(0);
    if (1 < nk) gload(1);
    pg_lds_barrier();
    for (int kt = 0; kt < nk; ++kt) {
        const uint32_t sb = (uint32_t)((kt & 1) * STAGEB);
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            u32x4 af[2], bf[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                af[i] = frag(sb + fa[i] + s * 16 * ROWB);
                bf[i] = frag(sb + fb[i] + s * 16 * ROWB);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = pg_mma(af[i], bf[j], acc[i][j]);
        }
        if (kt + 1 < nk) lstore((kt + 1) & 1);
        if (kt + 2 < nk) gload(kt + 2);
        pg_lds_barrier();
    }
}

template <class S>
__global__ __launch_bounds__(S::NTHR) void pgemm_kernel(const PlaneProblem *__restrict__ probs, int nprobs,
                                                        int total_tiles, const int *__restrict__ state)
{
    constexpr int NTA = S::NTA, NTB = S::NTB, WTM = S::WTM, WTN = S::WTN;
    constexpr int TM = S::TM, TN = S::TN, BK = S::BK;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    ASTERIA_LDS uint16_t *smem = (ASTERIA_LDS uint16_t *)smem_raw;

    const int per_xcd = (total_tiles + NUM_XCD - 1) / NUM_XCD;
    const int t_global = (int)(blockIdx.x % NUM_XCD) * per_xcd + (int)(blockIdx.x / NUM_XCD);
    if (t_global >= total_tiles) return;
    int plo = 0, phi = nprobs - 1;
    while (plo < phi) {
        const int mid = (plo + phi + 1) >> 1;
        if (probs[mid].tile_start <= t_global) plo = mid; else phi = mid - 1;
    }
    const PlaneProblem P = probs[plo];   // by value: the fields stay in scalar registers across the stores below
    if (P.state_idx >= 0) {
        const int st = state[P.state_idx];
        if (!((1 << st) & P.state_mask)) return;
    }
    const int lt = t_global - P.tile_start;
    const bool sym = (P.flags & GEMM_SYM) != 0;
    int ti, tj;
    if (sym) tri_decode(lt, ti, tj);
    else { ti = lt / P.tiles_n; tj = lt % P.tiles_n; }
    const int row0 = ti * TM, col0 = tj * TN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / S::WGN, wn = wave % S::WGN;
    const int r = lane & 31, h = lane >> 5;

    floatx16 acc[WTM][WTN];
#pragma unroll
    for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // ---- K loop ---------------------------------------------------------------------------------
    bool kmajor = false;
    if constexpr (S::KM) {
        kmajor = (P.flags & PG_KMAJOR) != 0;
        if (kmajor) pg_kmajor_loop<S>(acc, P, row0, col0, smem, tid, wm, wn, lane);
    }
    if (!kmajor) {
        PgLoader<S, S::FA, NTA, TM> la;
        PgLoader<S, S::FB, NTB, TN> lb;
        la.init(P.A, P.lda, row0, tid);
        lb.init(P.B, P.ldb, col0, tid);
        // fragments: lane (r, h) takes k = 8 h .. 8 h + 7 of k-step s, i.e. chunk (s / 2) * NT * 4 + t * 4 + (s % 2) * 2 + h
        const uint32_t lds_fa = (uint32_t)((wm * WTM * 32 + r) * S::ROW_A);
        const uint32_t lds_fb = (uint32_t)(TM * S::ROW_A + (wn * WTN * 32 + r) * S::ROW_B);
        const int swa = pg_swz<S::CPR_A>(r), swb = pg_swz<S::CPR_B>(r);
        constexpr int DEPTH = S::DEPTH;
        const int nk = (P.K + BK - 1) / BK;

        // DEPTH register sets: slab j waits in set j % DEPTH from its global load until it is
        // stored to LDS one iteration before use.
        auto gload = [&](auto setc, int slab) {
            constexpr int set = decltype(setc)::value;
            la.template gload<set>(slab);
            lb.template gload<set>(slab);
        };
        auto lstore = [&](auto setc, int stage) {
            constexpr int set = decltype(setc)::value;
            ASTERIA_LDS uint16_t *d = smem + stage * S::STAGE;
            la.template lstore<set>(d);
            lb.template lstore<set>(d + TM * S::ROW_A);
        };
        auto compute = [&](int cur) {
            const ASTERIA_LDS uint16_t *fa = smem + cur * S::STAGE + lds_fa;
            const ASTERIA_LDS uint16_t *fb = smem + cur * S::STAGE + lds_fb;
#pragma unroll
            for (int s = 0; s < S::STEPS; ++s) {
                u32x4 af[NTA][WTM], bf[NTB][WTN];
#pragma unroll
                for (int t = 0; t < NTA; ++t) {
                    const int ca = (((s / 2) * NTA + t) * S::CPG + (s % 2) * 2 + h) ^ swa;
#pragma unroll
                    for (int i = 0; i < WTM; ++i)
                        af[t][i] = *(const ASTERIA_LDS u32x4 *)(fa + i * 32 * S::ROW_A + ca * 8);
                }
#pragma unroll
                for (int t = 0; t < NTB; ++t) {
                    const int cb = (((s / 2) * NTB + t) * S::CPG + (s % 2) * 2 + h) ^ swb;
#pragma unroll
                    for (int j = 0; j < WTN; ++j)
                        bf[t][j] = *(const ASTERIA_LDS u32x4 *)(fb + j * 32 * S::ROW_B + cb * 8);
                }
                // small cross terms first, the leading product last
#pragma unroll
                for (int order = NTA + NTB - 2; order >= 0; --order)
#pragma unroll
                    for (int ta = 0; ta < NTA; ++ta) {
                        const int tb = order - ta;
                        if (tb < 0 || tb >= NTB) continue;
                        if (!((S::PAIRS >> (ta * 2 + tb)) & 1u)) continue;
#pragma unroll
                        for (int i = 0; i < WTM; ++i)
#pragma unroll
                            for (int j = 0; j < WTN; ++j) acc[i][j] = pg_mma(af[ta][i], bf[tb][j], acc[i][j]);
                    }
            }
        };
        // iteration kt: compute slab kt; store slab kt + 1 (set (kt + 1) % DEPTH) to the other
        // stage; refill that set with slab kt + 1 + DEPTH
        auto iteration = [&](auto setc, int kt) {
            compute(kt & 1);
            if (kt + 1 < nk) lstore(setc, (kt + 1) & 1);
            if (kt + 1 + DEPTH < nk) gload(setc, kt + 1 + DEPTH);
            pg_lds_barrier();
        };

        if constexpr (S::MODE == 1) {
            // Two groups of wavefronts (one wavefront of each per SIMD) run half a period apart:
            // while one group issues the MFMAs of a k-step from registers, the other reads its
            // next fragments from LDS and moves the next slab global -> LDS.  Every phase ends in
            // a workgroup barrier; the second group enters one barrier late and the first one
            // leaves one barrier late, so all wavefronts execute the same number of barriers.
            static_assert(DEPTH == 1 && (S::NTHR / 64) % 2 == 0, "alternating groups: one register set, even wavefront count");
            using Set0 = std::integral_constant<int, 0>;
            const int grp = __builtin_amdgcn_readfirstlane(wave) / (S::NTHR / 128);
            u32x4 af[NTA][WTM], bf[NTB][WTN];
            auto phase_barrier = [&]() {
                __builtin_amdgcn_sched_barrier(0);
                pg_lds_barrier();
                __builtin_amdgcn_sched_barrier(0);
            };
            gload(Set0{}, 0);
            lstore(Set0{}, 0);
            if (1 < nk) gload(Set0{}, 1);
            phase_barrier();
            if (grp == 1) phase_barrier();
            for (int kt = 0; kt < nk; ++kt) {
                const ASTERIA_LDS uint16_t *fa = smem + (kt & 1) * S::STAGE + lds_fa;
                const ASTERIA_LDS uint16_t *fb = smem + (kt & 1) * S::STAGE + lds_fb;
#pragma unroll
                for (int s = 0; s < S::STEPS; ++s) {
                    // load phase
#pragma unroll
                    for (int t = 0; t < NTA; ++t) {
                        const int ca = (((s / 2) * NTA + t) * S::CPG + (s % 2) * 2 + h) ^ swa;
#pragma unroll
                        for (int i = 0; i < WTM; ++i)
                            af[t][i] = *(const ASTERIA_LDS u32x4 *)(fa + i * 32 * S::ROW_A + ca * 8);
                    }
#pragma unroll
                    for (int t = 0; t < NTB; ++t) {
                        const int cb = (((s / 2) * NTB + t) * S::CPG + (s % 2) * 2 + h) ^ swb;
#pragma unroll
                        for (int j = 0; j < WTN; ++j)
                            bf[t][j] = *(const ASTERIA_LDS u32x4 *)(fb + j * 32 * S::ROW_B + cb * 8);
                    }
                    if (s == S::STEPS - 1) {
                        if (kt + 1 < nk) lstore(Set0{}, (kt + 1) & 1);
                        if (kt + 2 < nk) gload(Set0{}, kt + 2);
                    }
                    phase_barrier();
                    // multiply phase
                    __builtin_amdgcn_s_setprio(1);
#pragma unroll
                    for (int order = NTA + NTB - 2; order >= 0; --order)
#pragma unroll
                        for (int ta = 0; ta < NTA; ++ta) {
                            const int tb = order - ta;
                            if (tb < 0 || tb >= NTB) continue;
                            if (!((S::PAIRS >> (ta * 2 + tb)) & 1u)) continue;
#pragma unroll
                            for (int i = 0; i < WTM; ++i)
#pragma unroll
                                for (int j = 0; j < WTN; ++j) acc[i][j] = pg_mma(af[ta][i], bf[tb][j], acc[i][j]);
                        }
                    __builtin_amdgcn_s_setprio(0);
                    phase_barrier();
                }
            }
            if (grp == 0) phase_barrier();
        } else {
            gload(std::integral_constant<int, 0>{}, 0);
            if constexpr (DEPTH > 1) { if (1 < nk) gload(std::integral_constant<int, 1>{}, 1); }
            if constexpr (DEPTH > 2) { if (2 < nk) gload(std::integral_constant<int, 2>{}, 2); }
            lstore(std::integral_constant<int, 0>{}, 0);
            if (DEPTH < nk) gload(std::integral_constant<int, 0>{}, DEPTH);
            pg_lds_barrier();
            for (int kt0 = 0; kt0 < nk; kt0 += DEPTH) {
                // slab kt + 1 lives in set (kt + 1) % DEPTH
                if constexpr (DEPTH == 1) {
                    iteration(std::integral_constant<int, 0>{}, kt0);
                } else {
                    iteration(std::integral_constant<int, 1>{}, kt0);
                    if constexpr (DEPTH > 2) { if (kt0 + 1 < nk) iteration(std::integral_constant<int, 2>{}, kt0 + 1); }
                    if (kt0 + DEPTH - 1 < nk) iteration(std::integral_constant<int, 0>{}, kt0 + DEPTH - 1);
                }
            }
        }
    }

    // ---- epilogue: 128 x 128 quadrants through an fp32 LDS tile ----------------------------------
    const float alpha = P.alpha;
    ASTERIA_LDS float *ct = (ASTERIA_LDS float *)smem_raw;
    constexpr int CP = S::CT_PITCH;
    constexpr int QM = TM / 128, QN = TN / 128;
    constexpr int WROWS = WTM * 32, WCOLS = WTN * 32;     // wavefront sub-tile
    constexpr int ITEMS = 128 * 16 / S::NTHR;             // 8-column row pieces per thread
#pragma unroll 1
    for (int q = 0; q < QM * QN; ++q) {
        const int qi = q / QN, qj = q % QN;
        const int gi = ti * QM + qi, gj = tj * QN + qj;   // quadrant coordinates in units of 128
        if (gi * 128 >= P.M || gj * 128 >= P.N) continue;
        if (sym && gi < gj) continue;
        const bool diag = sym && gi == gj;
        // packed lower-tile output (tiles are 128 x 128, as the quadrants): nothing is stored above the diagonal
        const bool packed = (P.flags & GEMM_C_PACKED) != 0;
        const bool mirror = sym && gi > gj && !packed;
        float *ctile = packed ? P.C32 + (((size_t)gi * (gi + 1) / 2 + gj) * PACK_T * PACK_T) : nullptr;
        const bool store_t = !sym && (P.flags & GEMM_STORE_T) != 0;   // only the transposed image is stored
        // does this wavefront own part of the quadrant?
        const int wr0 = wm * WROWS - qi * 128, wc0 = wn * WCOLS - qj * 128;   // sub-tile origin relative to the quadrant
        const bool owns = wr0 < 128 && wr0 + WROWS > 0 && wc0 < 128 && wc0 + WCOLS > 0;
        for (int pass = store_t ? 1 : 0; pass < ((mirror || store_t) ? 2 : 1); ++pass) {
            if (owns) {
#pragma unroll
                for (int i = 0; i < WTM; ++i) {
                    const int br = wr0 + i * 32;
                    if (br < 0 || br >= 128) continue;
#pragma unroll
                    for (int j = 0; j < WTN; ++j) {
                        const int bc = wc0 + j * 32;
                        if (bc < 0 || bc >= 128) continue;
                        if (pass == 0) {
#pragma unroll
                            for (int v = 0; v < 16; ++v)
                                ct[(br + 8 * (v >> 2) + 4 * h + (v & 3)) * CP + bc + r] = alpha * acc[i][j][v];
                        } else {
                            // transposed: ct[col][row .. row + 3]
#pragma unroll
                            for (int g4 = 0; g4 < 4; ++g4) {
                                floatx4 w;
#pragma unroll
                                for (int e = 0; e < 4; ++e) w[e] = alpha * acc[i][j][4 * g4 + e];
                                *(ASTERIA_LDS floatx4 *)(ct + (bc + r) * CP + br + 8 * g4 + 4 * h) = w;
                            }
                        }
                    }
                }
            }
            __syncthreads();
            // pass 0 writes quadrant (gi, gj); pass 1 writes its mirror image at (gj, gi)
            const int orow0 = (pass == 0 ? gi : gj) * 128, ocol0 = (pass == 0 ? gj : gi) * 128;
#pragma unroll 2
            for (int it = 0; it < ITEMS; ++it) {
                const int item = tid + it * S::NTHR;
                const int lr = item >> 4, lc = (item & 15) * 8;
                float val[8];
                if (diag) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int c = lc + e;
                        val[e] = (lr >= c) ? ct[lr * CP + c] : ct[c * CP + lr];
                    }
                } else {
                    const floatx4 v0 = *(const ASTERIA_LDS floatx4 *)(ct + lr * CP + lc);
                    const floatx4 v1 = *(const ASTERIA_LDS floatx4 *)(ct + lr * CP + lc + 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) { val[e] = v0[e]; val[4 + e] = v1[e]; }
                }
                pg_emit(P, orow0 + lr, ocol0 + lc, pass == 0 ? P.M : P.N, pass == 0 ? P.N : P.M, val, ctile);
            }
            __syncthreads();
        }
    }
}

// 256 x 256 tiles, 8 wavefronts in two alternating groups, both operands plain fp32 matrices split
// into two bf16 terms while staged: the non-symmetric products of the precondition and of the SOAP
// rotations whose shapes fill whole tiles
using PgF32x2 = PgShape<2, 2, PG_PAIRS_2x2, 2, 4, 4, 2, 32, 1, 1, true, true>;

// a plain fp32 matrix can feed PgF32x2: 16-byte aligned rows, whole tiles and slabs
inline bool pg_f32_operand_ok(const void *p, int rows, int k, int ld)
{
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0 && (ld % 4) == 0 && (rows % PgF32x2::TM) == 0 &&
           (k % PgF32x2::BK) == 0;
}

inline int pg_tri_tiles(int n, int tile)
{
    const int t = (n + tile - 1) / tile;
    return t * (t + 1) / 2;
}

template <class S>
inline hipError_t launch_pgemm(const PlaneProblem *probs, int nprobs, int total_tiles, const int *state,
                               hipStream_t stream, int kind = 256)
{
    if (total_tiles <= 0 || nprobs <= 0) return hipSuccess;
    auto kern = pgemm_kernel<S>;
    static bool configured[MAX_DEVICES] = {};
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), S::LDS_BYTES, configured); e != hipSuccess) return e;
    const int per_xcd = (total_tiles + NUM_XCD - 1) / NUM_XCD;
    profile_begin(kind, stream);
    hipLaunchKernelGGL(kern, dim3(per_xcd * NUM_XCD), dim3(S::NTHR), S::LDS_BYTES, stream, probs, nprobs,
                       total_tiles, state);
    profile_end(stream);
    return hipGetLastError();
}

}  // namespace asteria
