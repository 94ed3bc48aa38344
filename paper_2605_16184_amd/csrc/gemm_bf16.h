// Grouped GEMM on the gfx950 bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// Same problem table, tile order and epilogue as gemm.h; operands are always k-contiguous.
// An operand is either bf16 in memory (used as is - bf16 x bf16 products are exact in fp32) or
// fp32 in memory and split on the fly into NT bf16 terms (x ~ hi + lo, hi = bf16(x),
// lo = bf16(x - hi)): with two terms per operand the kernel issues hi*hi, hi*lo and lo*hi, which
// keeps 16 to 18 bits of the fp32 operands at three bf16 MFMA passes.
//
// With F16 = true the two terms of an fp32 operand are fp16 instead of bf16 (v_mfma_f32_32x32x16_f16):
// 11 + 11 significant bits instead of 8 + 8, i.e. the operand to 2^-22, close to fp32, at the same
// three passes.  fp16 has a 5-bit exponent, so each operand is first multiplied by a power of two
// that brings its largest entries near the top of the fp16 range (the caller knows a bound) and the
// accumulators are divided by the product of the two scales afterwards; entries more than 2^-25 of
// the bound below it lose relative, not absolute, accuracy.
//
// Workgroup = 256 threads = 2 x 2 wavefronts of 64 x 64 (2 x 2 MFMA tiles each), K slabs of 64
// (32 when operands are split, to fit both terms of both operands in LDS twice).
#pragma once
#include "gemm.h"

#ifndef ASTERIA_BF16_MIN_WAVES
// wavefronts per SIMD the register budget is held to.  Two workgroups per CU; a third (168 registers,
// one LDS stage of 32 KiB and two barriers per slab) changed nothing: 219.6 against 218.3 TFLOP/s.
#define ASTERIA_BF16_MIN_WAVES 2
#endif
#ifndef ASTERIA_SPLIT_STAGES
#define ASTERIA_SPLIT_STAGES 2   // LDS stages of the products with both operands split
#endif
#ifndef ASTERIA_SPLIT_BK
#define ASTERIA_SPLIT_BK 32   // K slab of the products with both operands split: 64 KiB of LDS, two workgroups per CU (64: one workgroup, 218 -> 168 TFLOP/s)
#endif

namespace asteria {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct MmaBf16 {
    static constexpr int T = 32;
    static constexpr int NACC = 16;
    static constexpr int WAVES_M = 2, WAVES_N = 2;
    static constexpr int NTHR = 256;
    static constexpr int WTM = 2, WTN = 2;
    typedef floatx16 acc_t;
    __device__ static __forceinline__ acc_t mma(u32x4 a, u32x4 b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
    __device__ static __forceinline__ acc_t mma_f16(u32x4 a, u32x4 b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b),
                                                      c, 0, 0, 0);
    }
    __device__ static __forceinline__ int acc_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }
};

// hi / lo bf16 split of four fp32 values with round-to-nearest in both terms: hi = bf16(x),
// lo = bf16(x - hi) (that difference is exact in fp32), so hi + lo keeps x to 2^-18 relative.
// gfx950 converts two fp32 to a packed bf16 pair in one instruction (v_cvt_pk_bf16_f32), which
// makes this as cheap as a truncating split: per pair one convert, two unpacks, two subtracts,
// one convert.  The split runs once per tile and slab, so its cost competes with the MFMA work
// it feeds.  Returns packed pairs.
__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float floatx2_t __attribute__((ext_vector_type(2)));
    const floatx2_t f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

__device__ __forceinline__ void split4(u32x4 x, u32x2 &hi, u32x2 &lo, bool want_lo)
{
    const float x0 = __uint_as_float(x[0]), x1 = __uint_as_float(x[1]);
    const float x2 = __uint_as_float(x[2]), x3 = __uint_as_float(x[3]);
    hi[0] = cvt_pk_bf16(x0, x1);
    hi[1] = cvt_pk_bf16(x2, x3);
    if (want_lo) {
        const float d0 = x0 - __uint_as_float(hi[0] << 16), d1 = x1 - __uint_as_float(hi[0] & 0xffff0000u);
        const float d2 = x2 - __uint_as_float(hi[1] << 16), d3 = x3 - __uint_as_float(hi[1] & 0xffff0000u);
        lo[0] = cvt_pk_bf16(d0, d1);
        lo[1] = cvt_pk_bf16(d2, d3);
    } else {
        lo[0] = 0u; lo[1] = 0u;
    }
}

// the same split into two fp16 terms of x * scale (round to nearest in both)
__device__ __forceinline__ void split4_f16(u32x4 x, u32x2 &hi, u32x2 &lo, float scale)
{
    typedef _Float16 halfx2_t __attribute__((ext_vector_type(2)));
    typedef float floatx2_t __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const floatx2_t v = {__uint_as_float(x[2 * e]) * scale, __uint_as_float(x[2 * e + 1]) * scale};
        const halfx2_t h = __builtin_convertvector(v, halfx2_t);
        const floatx2_t d = v - __builtin_convertvector(h, floatx2_t);
        hi[e] = __builtin_bit_cast(uint32_t, h);
        lo[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(d, halfx2_t));
    }
}

// One operand tile (128 rows x BK) of input type TI staged as bf16 (or fp16) terms in LDS.
template <typename TI, int NT, int BK, bool F16 = false>
struct Bf16Stage {
    static_assert(!F16 || sizeof(TI) == 4, "fp16 terms: fp32 source");
    static constexpr int EPV = Elem<TI>::EPV;              // 8 (bf16) or 4 (fp32) elements per 16 bytes
    static constexpr int VPR = BK / EPV;
    static constexpr int NV = BM * VPR / 256;
    // LDS rows are unpadded (BK elements); the 16-byte chunks of a row are XOR-swizzled by the row
    // index instead: the loader's lanes then write whole contiguous rows (4 rows = 256 bytes = all
    // 64 banks per 32 lanes), and the 16 rows a quarter-wavefront reads for one fragment chunk fall
    // into 16 distinct 16-byte bank groups.  (A 16-byte pad per row made the 8-byte stores of the
    // split terms collide two ways: a third of the LDS cycles of this kernel were conflicts.)
    static constexpr int PITCH = BK;
    static constexpr int CPR = BK / 8;                     // 16-byte chunks per row
    __device__ static __forceinline__ int swz(int row) { return (row / (16 / CPR)) % CPR; }
    static_assert(CPR == 4 || CPR == 8, "swizzle geometry");
    static constexpr int TERM_ELEMS = BM * PITCH;
    static constexpr int LDS_ELEMS = NT * TERM_ELEMS;      // per stage
    static_assert(NV >= 1, "slab too small");
    static_assert(sizeof(TI) == 2 ? NT == 1 : true, "bf16 operands are exact: one term");

    u32x4 r[NV];

    template <bool GUARD>
    __device__ __forceinline__ void load(const TI *base, int ld, int row0, int rows, int k0, int k_left,
                                         bool vec_ok, int tid)
    {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int idx = tid + 256 * v;
            const int a = idx / VPR, b = idx % VPR;
            const TI *p = base + (size_t)(row0 + a) * ld + k0 + b * EPV;
            if (!GUARD) r[v] = *(const ASTERIA_GLOBAL u32x4 *)(p);
            else r[v] = load16<TI>(p, (a < rows) ? (k_left - b * EPV) : 0, vec_ok);
        }
    }

    __device__ __forceinline__ void store(ASTERIA_LDS uint16_t *lds, int tid, float scale = 1.0f) const
    {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int idx = tid + 256 * v;
            const int a = idx / VPR, b = idx % VPR;
            // bf16 source: vector b is chunk b; fp32 source: vector b is half (b % 2) of chunk b / 2
            const int chunk = (sizeof(TI) == 2) ? b : (b >> 1);
            ASTERIA_LDS uint16_t *dst = lds + a * PITCH + ((chunk ^ swz(a)) << 3) + ((sizeof(TI) == 2) ? 0 : (b & 1) * 4);
            if (sizeof(TI) == 2) {
                *(ASTERIA_LDS u32x4 *)dst = r[v];
            } else {
                u32x2 hi, lo;
                if (F16) split4_f16(r[v], hi, lo, scale);
                else split4(r[v], hi, lo, NT == 2);
                *(ASTERIA_LDS u32x2 *)dst = hi;
                if (NT == 2) *(ASTERIA_LDS u32x2 *)(dst + TERM_ELEMS) = lo;
            }
        }
    }
};

// TRI: which 32 x 32 blocks (i, j) of the wavefront's 64 x 64 sub-tile are multiplied (TRI_ALL,
// TRI_NONE, or those with j - i <= TRI), as in gemm_mainloop
template <typename TA, typename TB, int NTA, int NTB, bool GUARD, int TRI = TRI_ALL, bool F16 = false>
__device__ __forceinline__ void gemm_bf16_mainloop(floatx16 (&acc)[2][2], const TA *Ab, const TB *Bb, int lda,
                                                   int ldb, int row0, int col0, int rowsA, int rowsB, int K,
                                                   bool vecA, bool vecB, ASTERIA_LDS uint16_t *smem, int tid,
                                                   int wm, int wn, int r, int h, float sca = 1.0f, float scb = 1.0f)
{
    constexpr int BK = (NTA + NTB > 2) ? ASTERIA_SPLIT_BK : 64;
    using StA = Bf16Stage<TA, NTA, BK, F16>;
    using StB = Bf16Stage<TB, NTB, BK, F16>;
    auto mma = [](u32x4 a, u32x4 b, floatx16 c) __attribute__((always_inline)) {
        return F16 ? MmaBf16::mma_f16(a, b, c) : MmaBf16::mma(a, b, c);
    };
    constexpr int KPL = BK / 2;          // k values per lane half and slab
    constexpr int STEPS = KPL / 8;       // MFMA k-steps per slab (8 bf16 per lane and step)
    StA sa;
    StB sb;
    constexpr int STAGES = (NTA + NTB > 2) ? ASTERIA_SPLIT_STAGES : 2;
    ASTERIA_LDS uint16_t *const smemB = smem + STAGES * StA::LDS_ELEMS;
    const int nk = (K + BK - 1) / BK;
    sa.template load<GUARD>(Ab, lda, row0, rowsA, 0, K, vecA, tid);
    sb.template load<GUARD>(Bb, ldb, col0, rowsB, 0, K, vecB, tid);
    sa.store(smem, tid, sca);
    sb.store(smemB, tid, scb);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = STAGES == 2 ? (kt & 1) : 0;
        if (kt + 1 < nk) {
            const int k0 = (kt + 1) * BK;
            sa.template load<GUARD>(Ab, lda, row0, rowsA, k0, K - k0, vecA, tid);
            sb.template load<GUARD>(Bb, ldb, col0, rowsB, k0, K - k0, vecB, tid);
        }
        const ASTERIA_LDS uint16_t *as = smem + cur * StA::LDS_ELEMS;
        const ASTERIA_LDS uint16_t *bs = smemB + cur * StB::LDS_ELEMS;
#pragma unroll
        for (int s = 0; s < (TRI == TRI_NONE ? 0 : STEPS); ++s) {
            const int ck = h * (KPL / 8) + s;    // the lane half owns a contiguous k range of the slab: chunk index
            u32x4 ah[2], al[2], bh[2], bl[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int rr = wm * 64 + i * 32 + r;
                const int kk = (ck ^ StA::swz(rr)) << 3;
                ah[i] = *(const ASTERIA_LDS u32x4 *)(as + rr * StA::PITCH + kk);
                if (NTA == 2) al[i] = *(const ASTERIA_LDS u32x4 *)(as + StA::TERM_ELEMS + rr * StA::PITCH + kk);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int cc = wn * 64 + j * 32 + r;
                const int kk = (ck ^ StB::swz(cc)) << 3;
                bh[j] = *(const ASTERIA_LDS u32x4 *)(bs + cc * StB::PITCH + kk);
                if (NTB == 2) bl[j] = *(const ASTERIA_LDS u32x4 *)(bs + StB::TERM_ELEMS + cc * StB::PITCH + kk);
            }
            // small cross terms first, the leading product last
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if (TRI != TRI_ALL && j - i > TRI) continue;
                    if (NTA == 2) acc[i][j] = mma(al[i], bh[j], acc[i][j]);
                    if (NTB == 2) acc[i][j] = mma(ah[i], bl[j], acc[i][j]);
                }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    if (TRI == TRI_ALL || j - i <= TRI) acc[i][j] = mma(ah[i], bh[j], acc[i][j]);
        }
        if (STAGES == 1) __syncthreads();      // every wavefront has read the slab before it is overwritten
        if (kt + 1 < nk) {
            const int nxt = STAGES == 2 ? (cur ^ 1) : 0;
            sa.store(smem + nxt * StA::LDS_ELEMS, tid, sca);
            sb.store(smemB + nxt * StB::LDS_ELEMS, tid, scb);
        }
        __syncthreads();
    }
}

template <typename TA, typename TB, int NTA, int NTB, bool F16 = false>
__global__ __launch_bounds__(256, ASTERIA_BF16_MIN_WAVES) void gemm_bf16_grouped_kernel(const GemmProblem *__restrict__ probs, int nprobs,
                                                                int total_tiles, const int *__restrict__ state)
{
    using MM = MmaBf16;
    constexpr int BK = (NTA + NTB > 2) ? ASTERIA_SPLIT_BK : 64;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    ASTERIA_LDS uint16_t *smem = (ASTERIA_LDS uint16_t *)smem_raw;
    // the reduction scratch of the epilogue reuses the operand buffer (free after the K loop): with
    // no static LDS two workgroups of the split variants (64 KiB each) fit one CU's 160 KiB
    float *red = reinterpret_cast<float *>(smem_raw);

    const int per_xcd = (total_tiles + NUM_XCD - 1) / NUM_XCD;
    const int t_global = (int)(blockIdx.x % NUM_XCD) * per_xcd + (int)(blockIdx.x / NUM_XCD);
    if (t_global >= total_tiles) return;
    int lo = 0, hi = nprobs - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (probs[mid].tile_start <= t_global) lo = mid; else hi = mid - 1;
    }
    const GemmProblem &P = probs[lo];
    if (P.state_idx >= 0) {
        const int st = state[P.state_idx];
        if (!((1 << st) & P.state_mask)) return;
    }
    const int lt = t_global - P.tile_start;
    int ti, tj;
    if (P.flags & GEMM_SYM) tri_decode(lt, ti, tj);
    else { ti = lt / P.tiles_n; tj = lt % P.tiles_n; }
    const int M = P.M, N = P.N, K = P.K;
    const int row0 = ti * BM, col0 = tj * BN;
    const int rowsA = min(BM, M - row0), rowsB = min(BN, N - col0);
    const TA *Ab = reinterpret_cast<const TA *>(P.A);
    const TB *Bb = reinterpret_cast<const TB *>(P.B);
    const int lda = P.lda, ldb = P.ldb;
    const bool vecA = ((reinterpret_cast<uintptr_t>(Ab) & 15u) == 0) && ((((size_t)lda * sizeof(TA)) & 15u) == 0);
    const bool vecB = ((reinterpret_cast<uintptr_t>(Bb) & 15u) == 0) && ((((size_t)ldb * sizeof(TB)) & 15u) == 0);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 31, h = lane >> 5;

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const bool fast = vecA && vecB && rowsA == BM && rowsB == BN && (K % BK) == 0;
    // diagonal tile of a symmetric product: blocks wholly above the diagonal are never stored and
    // are not multiplied; the wavefront at (wm, wn) keeps the blocks with j - i <= 2 (wm - wn)
    int d = 2;
    if ((P.flags & GEMM_SYM) && ti == tj) {
        const int w = __builtin_amdgcn_readfirstlane(wave);
        d = 2 * ((w >> 1) - (w & 1));
    }
    // fp16 terms: the operands are scaled into the fp16 range before the split, the sums scaled back
    float sca = 1.0f, scb = 1.0f;
    if (F16) { sca = P.sa_dev ? *P.sa_dev : P.sa; scb = P.sb_dev ? *P.sb_dev : P.sb; }
    if (fast && d == 0)
        gemm_bf16_mainloop<TA, TB, NTA, NTB, false, 0, F16>(acc, Ab, Bb, lda, ldb, row0, col0, rowsA, rowsB, K, vecA,
                                                            vecB, smem, tid, wm, wn, r, h, sca, scb);
    else if (fast && d < 0)
        gemm_bf16_mainloop<TA, TB, NTA, NTB, false, TRI_NONE, F16>(acc, Ab, Bb, lda, ldb, row0, col0, rowsA, rowsB, K,
                                                                   vecA, vecB, smem, tid, wm, wn, r, h, sca, scb);
    else if (fast)
        gemm_bf16_mainloop<TA, TB, NTA, NTB, false, TRI_ALL, F16>(acc, Ab, Bb, lda, ldb, row0, col0, rowsA, rowsB, K,
                                                                  vecA, vecB, smem, tid, wm, wn, r, h, sca, scb);
    else
        gemm_bf16_mainloop<TA, TB, NTA, NTB, true, TRI_ALL, F16>(acc, Ab, Bb, lda, ldb, row0, col0, rowsA, rowsB, K,
                                                                 vecA, vecB, smem, tid, wm, wn, r, h, sca, scb);
    if (F16) {
        const float inv = 1.0f / (sca * scb);     // powers of two: exact
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] *= inv;
    }
    gemm_epilogue<MM, float>(P, acc, lt, ti, tj, row0, col0, rowsA, rowsB, wm, wn, r, h, lane, wave, tid, red);
}

template <typename TA, typename TB, int NTA, int NTB, bool F16 = false>
inline hipError_t launch_gemm_bf16_grouped(const GemmProblem *probs, int nprobs, int total_tiles,
                                           const int *state, hipStream_t stream)
{
    if (total_tiles <= 0 || nprobs <= 0) return hipSuccess;
    constexpr int BK = (NTA + NTB > 2) ? ASTERIA_SPLIT_BK : 64;
    auto kern = gemm_bf16_grouped_kernel<TA, TB, NTA, NTB, F16>;
    constexpr size_t lds = sizeof(uint16_t) * ((NTA + NTB > 2) ? ASTERIA_SPLIT_STAGES : 2) *
                           (size_t)(Bf16Stage<TA, NTA, BK>::LDS_ELEMS + Bf16Stage<TB, NTB, BK>::LDS_ELEMS);
    static bool configured[MAX_DEVICES] = {};
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds, configured); e != hipSuccess) return e;
    const int per_xcd = (total_tiles + NUM_XCD - 1) / NUM_XCD;
    constexpr int kind = 32 | (sizeof(TA) == 2 ? 2 : 0) | (sizeof(TB) == 2 ? 4 : 0) | (NTA == 2 ? 64 : 0) | (NTB == 2 ? 128 : 0);
    profile_begin(kind, stream);
    hipLaunchKernelGGL(kern, dim3(per_xcd * NUM_XCD), dim3(256), lds, stream, probs, nprobs, total_tiles, state);
    profile_end(stream);
    return hipGetLastError();
}

}  // namespace asteria
