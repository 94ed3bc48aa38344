// Grouped GEMM core on the gfx950 matrix cores (fp32 and fp64 MFMA).
//
// One launch processes a device-resident table of independent problems
//     C = alpha * A' * B'^T + beta * C          (A' is M x K, B' is N x K)
// where each operand is either "k-contiguous" (element (r, k) at base[r * ld + k]) or
// "k-major" (element (r, k) at base[k * ld + r]).  With symmetric commuting operands
// (every product of the coupled root iteration, and G G^T / G^T G) only tiles on or below
// the diagonal are computed and the result is mirrored, so the output is exactly symmetric.
//
// Workgroup = 512 threads = 8 wavefronts, macro-tile 128 x 128 (fp32: 2 x 4 wavefronts of
// 64 x 32; fp64: 4 x 2 wavefronts of 32 x 64 - eight wavefronts keep the accumulators small enough
// for two workgroups per CU).  K is walked in slabs of BK staged through LDS (two stages,
// register prefetch of the next slab while the current one feeds the MFMA pipe).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace asteria {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef double doublex4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16-byte vector without class semantics

struct bf16_t { uint16_t bits; };

// Explicit address spaces: pointers that come out of a table or a runtime-indexed array are
// "generic" to the compiler, which then emits FLAT instructions; FLAT accesses count against
// both the vector-memory and the LDS wait counters and serialise the K loop.
#define ASTERIA_GLOBAL __attribute__((address_space(1)))
#define ASTERIA_LDS __attribute__((address_space(3)))

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// round-to-nearest-even, NaN kept quiet
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

enum : int {
    GEMM_SYM = 1,        // compute tiles with ti >= tj only, mirror the result
    GEMM_EPI_ROOT = 2,   // C2 = ep_a * I - ep_g * C ; partial[tile] = sum (C - I)^2
    GEMM_C_BF16 = 4,     // C is stored as bf16 (fp32 compute only)
    GEMM_STORE_T = 8,    // C is stored transposed: element (row, col) at C[col * ldc + row] (no beta, not symmetric)
    GEMM_C_F32 = 16,     // C is stored as fp32 (fp64 compute only): read, combined in fp64, rounded once
    GEMM_EPI_HANDOVER = 32,  // root epilogue of the last fp64 iteration: C and C2 are not stored (nothing reads the
                             // fp64 M and T again), C goes to C4 in fp32 instead (C3, the fp32 T, as usual)
    GEMM_C_PACKED = 64   // symmetric C in packed lower-tile storage (see packed_off); ldc unused, nothing above the diagonal tiles
};

// Packed lower-tile storage of a symmetric n x n fp32 matrix: the 128 x 128 tiles on and below the
// diagonal, tile (ti, tj), tj <= ti, at tile index ti (ti + 1) / 2 + tj, each tile dense row-major
// (diagonal tiles hold both of their triangles; the last tile row / column of a ragged n is padded,
// the padding is never read).  Every tile row is 512 bytes, so all accesses stay 16-byte aligned.
constexpr int PACK_T = 128;
__host__ __device__ inline size_t packed_tiles(int n) { const size_t t = (size_t)((n + PACK_T - 1) / PACK_T); return t * (t + 1) / 2; }
__host__ __device__ inline size_t packed_elems(int n) { return packed_tiles(n) * PACK_T * PACK_T; }
// offset of element (row, col); the tile of (row, col) must be on or below the diagonal
__host__ __device__ inline size_t packed_off(int row, int col)
{
    const size_t ti = (size_t)(row / PACK_T), tj = (size_t)(col / PACK_T);
    return ((ti * (ti + 1) / 2 + tj) * PACK_T + (size_t)(row % PACK_T)) * PACK_T + (size_t)(col % PACK_T);
}

struct GemmProblem {
    const void *A;
    const void *B;
    void *C;
    void *C2;
    float *C3;          // root epilogue: optional fp32 copy of C2
    float *C4;          // root epilogue with GEMM_EPI_HANDOVER: fp32 copy of C
    float *partial;
    const float *coef;  // root epilogue: device pointer to (a, g), or null to use ep_a / ep_g
    const float *sa_dev; // fp16-split kernel: device pointer to the scale of operand A, or null to use sa
    const float *sb_dev; // the same for operand B (null: sb)
    const int *gate;     // optional: the problem runs only while *gate == 0
    int M, N, K;
    int lda, ldb, ldc, ldc2, ldc3, ldc4;
    int tile_start;  // id of this problem's first tile within the launch
    int tiles_n;     // tile columns (non-symmetric problems)
    int state_idx;   // index into the launch's state[] array, or -1
    int state_mask;  // problem runs iff (1 << state[state_idx]) & state_mask
    float alpha, beta;
    float ep_a, ep_g;
    int flags;
    float sa, sb;       // fp16-split kernel: powers of two the operands are multiplied by before the split
};

// Measurement aid (see asteria_profile_enable): bracket a launch with HIP events on its stream.
void profile_begin(int kind, hipStream_t stream);
void profile_end(hipStream_t stream);
// While recording: device array of 3 doubles in which the int8 decision kernel adds up the algorithmic
// flops of the products it sends to the fp64 cores [0], to 4 slices [1] and to 5 slices [2]; else null.
double *profile_i8_counters();

// The dynamic-LDS limit of a kernel is an attribute per device: a launcher remembers, per device,
// that it has raised it (`done` is the launcher's own static array).
constexpr int MAX_DEVICES = 64;
inline hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes, bool (&done)[MAX_DEVICES])
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    if (!done[dev]) {
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return e;
        done[dev] = true;
    }
    return hipSuccess;
}

constexpr int BM = 128;
constexpr int BN = 128;
constexpr int NUM_XCD = 8;

// ---- per-precision matrix-core traits -------------------------------------------------------
template <typename TC> struct Mma;

// v_mfma_f32_32x32x2_f32: A[i][k] in lane i + 32 k, B[k][j] in lane j + 32 k,
// D[i][j] in lane j + 32 ((i / 4) % 2), register 4 (i / 8) + i % 4.
template <> struct Mma<float> {
    static constexpr int T = 32;       // MFMA tile edge
    static constexpr int KG = 2;       // lane groups along k
    static constexpr int NACC = 16;    // accumulator values per lane per tile
    static constexpr int BK = 32;      // K slab
    static constexpr int KPL = BK / KG;  // k values one lane consumes per slab
#ifndef ASTERIA_F32_WAVES_M
#define ASTERIA_F32_WAVES_M 2
#define ASTERIA_F32_WAVES_N 4
#endif
    static constexpr int WAVES_M = ASTERIA_F32_WAVES_M, WAVES_N = ASTERIA_F32_WAVES_N;   // wavefront grid over the 128 x 128 tile
    static constexpr int NTHR = 64 * WAVES_M * WAVES_N;
    static constexpr int WTM = 128 / WAVES_M / T;              // MFMA tiles per wavefront, rows (64 / 32)
    static constexpr int WTN = 128 / WAVES_N / T;              // MFMA tiles per wavefront, columns
    static constexpr int CH = 4;       // elements per 16-byte LDS chunk
    static constexpr int MIN_WAVES = 4;       // wavefronts per SIMD the register budget is held to: two workgroups per CU
    // slabs of global loads in flight ahead of the one being multiplied (2 needs a second register
    // set, which does not fit the budget above without spills, and gained 1 %)
    static constexpr int PREFETCH = 1;
    static constexpr int PITCH_KC = BK + 4;   // k-contiguous LDS row pitch (144 B)
    static constexpr int PITCH_KM = BM + 4;   // k-major LDS row pitch
    typedef floatx16 acc_t;
    __device__ static __forceinline__ acc_t mma(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    __device__ static __forceinline__ int acc_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }
};

// v_mfma_f64_16x16x4_f64: A[i][k] in lane i + 16 k, B[k][j] in lane j + 16 k,
// D[i][j] in lane j + 16 (i % 4), register i / 4.
template <> struct Mma<double> {
    static constexpr int T = 16;
    static constexpr int KG = 4;
    static constexpr int NACC = 4;
    static constexpr int BK = 16;
    static constexpr int KPL = BK / KG;
#ifndef ASTERIA_F64_WAVES_M
#define ASTERIA_F64_WAVES_M 4
#define ASTERIA_F64_WAVES_N 2
#endif
    static constexpr int WAVES_M = ASTERIA_F64_WAVES_M, WAVES_N = ASTERIA_F64_WAVES_N;
    static constexpr int NTHR = 64 * WAVES_M * WAVES_N;
    static constexpr int WTM = 128 / WAVES_M / T;
    static constexpr int WTN = 128 / WAVES_N / T;
    static constexpr int CH = 2;
    // wavefronts per SIMD the register budget is held to: one 8-wavefront workgroup per CU (a
    // budget for two spills the staged operands inside the K loop: 30 instead of 52 TFLOP/s)
    static constexpr int MIN_WAVES = 2;
    static constexpr int PREFETCH = 2;        // slabs of global loads in flight ahead of the one being multiplied
    static constexpr int PITCH_KC = BK + 2;   // 144 B
    static constexpr int PITCH_KM = BM + 2;
    typedef doublex4 acc_t;
    __device__ static __forceinline__ acc_t mma(double a, double b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    __device__ static __forceinline__ int acc_row(int v, int h) { return 4 * v + h; }
};

// ---- global -> register staging -------------------------------------------------------------
template <typename TI> struct Elem;
template <> struct Elem<float>  { static constexpr int EPV = 4; };
template <> struct Elem<double> { static constexpr int EPV = 2; };
template <> struct Elem<bf16_t> { static constexpr int EPV = 8; };

// 16 bytes starting at p; elements at index >= valid are zero.  vec_ok: p is 16-byte aligned.
template <typename TI>
__device__ __forceinline__ u32x4 load16(const TI *p, int valid, bool vec_ok)
{
    constexpr int EPV = Elem<TI>::EPV;
    union { u32x4 v; TI e[EPV]; } u;
    if (valid >= EPV && vec_ok) {
        u.v = *(const ASTERIA_GLOBAL u32x4 *)(p);
    } else {
        u.v = (u32x4){0u, 0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < EPV; ++e)
            if (e < valid) u.e[e] = p[e];
    }
    return u.v;
}

// write the EPV elements of one staged vector to LDS as TC, contiguous at dst
template <typename TC, typename TI> struct StoreLds;
template <> struct StoreLds<float, float> {
    __device__ static __forceinline__ void run(ASTERIA_LDS float *dst, u32x4 v) { *(ASTERIA_LDS u32x4 *)(dst) = v; }
};
template <> struct StoreLds<double, double> {
    __device__ static __forceinline__ void run(ASTERIA_LDS double *dst, u32x4 v) { *(ASTERIA_LDS u32x4 *)(dst) = v; }
};
template <> struct StoreLds<double, float> {   // fp32 data accumulated on the fp64 matrix cores
    __device__ static __forceinline__ void run(ASTERIA_LDS double *dst, u32x4 v)
    {
        typedef double doublex2 __attribute__((ext_vector_type(2)));
        doublex2 a, b;
        a[0] = (double)__uint_as_float(v[0]); a[1] = (double)__uint_as_float(v[1]);
        b[0] = (double)__uint_as_float(v[2]); b[1] = (double)__uint_as_float(v[3]);
        ((ASTERIA_LDS doublex2 *)dst)[0] = a;
        ((ASTERIA_LDS doublex2 *)dst)[1] = b;
    }
};
template <> struct StoreLds<double, bf16_t> {  // bf16 data accumulated on the fp64 matrix cores
    __device__ static __forceinline__ void run(ASTERIA_LDS double *dst, u32x4 v)
    {
        typedef double doublex2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            doublex2 a;
            a[0] = (double)__uint_as_float(v[w] << 16);
            a[1] = (double)__uint_as_float(v[w] & 0xffff0000u);
            ((ASTERIA_LDS doublex2 *)dst)[w] = a;
        }
    }
};
template <> struct StoreLds<float, bf16_t> {
    __device__ static __forceinline__ void run(ASTERIA_LDS float *dst, u32x4 v)
    {
        u32x4 lo, hi;
        lo.x = v.x << 16; lo.y = v.x & 0xffff0000u; lo.z = v.y << 16; lo.w = v.y & 0xffff0000u;
        hi.x = v.z << 16; hi.y = v.z & 0xffff0000u; hi.z = v.w << 16; hi.w = v.w & 0xffff0000u;
        ((ASTERIA_LDS u32x4 *)dst)[0] = lo;
        ((ASTERIA_LDS u32x4 *)dst)[1] = hi;
    }
};

// One operand tile (128 rows x BK) staged per thread as NV 16-byte vectors.
template <typename TC, typename TI, bool KMAJOR>
struct OperandStage {
    static constexpr int EPV = Elem<TI>::EPV;
    static constexpr int BK = Mma<TC>::BK;
    static constexpr int VPR = KMAJOR ? (BM / EPV) : (BK / EPV);       // vectors per stored row
    static constexpr int NTHREADS = Mma<TC>::NTHR;
    static constexpr int TOTAL = (KMAJOR ? BK : BM) * VPR;             // vectors per tile
    static constexpr int NV = (TOTAL + NTHREADS - 1) / NTHREADS;       // vectors per thread
    // a tile with fewer vectors than threads (bf16 data under the 16-wide fp64 slab): the threads
    // beyond the tile stage nothing
    static constexpr bool PARTIAL = (TOTAL % NTHREADS) != 0;
    static constexpr int LDS_ELEMS = KMAJOR ? BK * Mma<TC>::PITCH_KM : BM * Mma<TC>::PITCH_KC;

    u32x4 r[NV];

    // rows: number of valid rows of this tile (<= 128); k_left: valid k from k0 on.
    // GUARD = false: the tile is full, the slab is full and every vector is 16-byte aligned.
    template <bool GUARD>
    __device__ __forceinline__ void load(const TI *base, int ld, int row0, int rows, int k0, int k_left,
                                         bool vec_ok, int tid)
    {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int idx = tid + NTHREADS * v;
            const int a = idx / VPR;   // stored row
            const int b = idx % VPR;   // vector within the stored row
            if (PARTIAL && idx >= TOTAL) { r[v] = (u32x4){0u, 0u, 0u, 0u}; continue; }
            if (!GUARD) {
                const TI *p = KMAJOR ? base + (size_t)(k0 + a) * ld + row0 + b * EPV
                                     : base + (size_t)(row0 + a) * ld + k0 + b * EPV;
                r[v] = *(const ASTERIA_GLOBAL u32x4 *)(p);
            } else if (KMAJOR) {
                // stored row = k, vector runs along the tile's rows
                const int valid = (a < k_left) ? (rows - b * EPV) : 0;
                const TI *p = base + (size_t)(k0 + a) * ld + row0 + b * EPV;
                r[v] = load16<TI>(p, valid, vec_ok);
            } else {
                const int valid = (a < rows) ? (k_left - b * EPV) : 0;
                const TI *p = base + (size_t)(row0 + a) * ld + k0 + b * EPV;
                r[v] = load16<TI>(p, valid, vec_ok);
            }
        }
    }

    __device__ __forceinline__ void store(ASTERIA_LDS TC *lds, int tid) const
    {
        constexpr int PITCH = KMAJOR ? Mma<TC>::PITCH_KM : Mma<TC>::PITCH_KC;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int idx = tid + NTHREADS * v;
            const int a = idx / VPR;
            const int b = idx % VPR;
            if (PARTIAL && idx >= TOTAL) continue;
            StoreLds<TC, TI>::run(lds + a * PITCH + b * EPV, r[v]);
        }
    }
};

// ---- tile id decoding -------------------------------------------------------------------------
__device__ __forceinline__ void tri_decode(int t, int &ti, int &tj)
{
    // largest ti with ti (ti + 1) / 2 <= t
    int i = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
    while ((i + 1) * (i + 2) / 2 <= t) ++i;
    while (i * (i + 1) / 2 > t) --i;
    ti = i;
    tj = t - i * (i + 1) / 2;
}

template <typename TC> __device__ __forceinline__ TC load_c(const void *C, size_t off, int flags);
template <> __device__ __forceinline__ float load_c<float>(const void *C, size_t off, int flags)
{
    if (flags & GEMM_C_BF16) return bf16_to_f32(reinterpret_cast<const uint16_t *>(C)[off]);
    return reinterpret_cast<const float *>(C)[off];
}
template <> __device__ __forceinline__ double load_c<double>(const void *C, size_t off, int flags)
{
    if (flags & GEMM_C_F32) return (double)reinterpret_cast<const float *>(C)[off];
    return reinterpret_cast<const double *>(C)[off];
}
template <typename TC> __device__ __forceinline__ void store_c(void *C, size_t off, TC v, int flags);
template <> __device__ __forceinline__ void store_c<float>(void *C, size_t off, float v, int flags)
{
    if (flags & GEMM_C_BF16) reinterpret_cast<uint16_t *>(C)[off] = f32_to_bf16(v);
    else reinterpret_cast<float *>(C)[off] = v;
}
template <> __device__ __forceinline__ void store_c<double>(void *C, size_t off, double v, int flags)
{
    if (flags & GEMM_C_F32) reinterpret_cast<float *>(C)[off] = (float)v;
    else reinterpret_cast<double *>(C)[off] = v;
}

// K loop of one 128 x 128 tile: two LDS stages, the next slab is fetched into registers while
// the current one feeds the matrix cores.
// TRI selects which MFMA blocks (i, j) of the wavefront's sub-tile are multiplied: TRI_ALL all,
// TRI_NONE none (the wavefront still stages its share of the operands), any other value d the
// blocks with j - i <= d.  In a diagonal tile of a symmetric product the blocks wholly above the
// diagonal are never stored; for the wavefront at (wm, wn) those are the blocks with
// j - i > d = (wm WROWS - wn WCOLS) / T.
constexpr int TRI_ALL = 1000, TRI_NONE = -1000;
template <typename TC, typename TA, typename TB, bool AKM, bool BKM, bool GUARD, int TRI = TRI_ALL>
__device__ __forceinline__ void gemm_mainloop(typename Mma<TC>::acc_t (&acc)[Mma<TC>::WTM][Mma<TC>::WTN],
                                              const TA *Ab, const TB *Bb, int lda, int ldb, int row0, int col0,
                                              int rowsA, int rowsB, int K, bool vecA, bool vecB,
                                              ASTERIA_LDS TC *smem,
                                              int tid, int wm, int wn, int r, int h)
{
    using MM = Mma<TC>;
    constexpr int BK = MM::BK;
    constexpr int WTM = MM::WTM, WTN = MM::WTN;
    constexpr int WROWS = BM / MM::WAVES_M, WCOLS = BN / MM::WAVES_N;
    constexpr int T = MM::T;
    using StA = OperandStage<TC, TA, AKM>;
    using StB = OperandStage<TC, TB, BKM>;
    // LDS map: A stage 0 | A stage 1 | B stage 0 | B stage 1
    ASTERIA_LDS TC *const smemB = smem + 2 * StA::LDS_ELEMS;
    const int nk = (K + BK - 1) / BK;
    auto compute = [&](int cur) {
        const ASTERIA_LDS TC *as = smem + cur * StA::LDS_ELEMS;
        const ASTERIA_LDS TC *bs = smemB + cur * StB::LDS_ELEMS;
        // lane group h consumes k = h * KPL .. h * KPL + KPL - 1 of the slab, the same for A and B
#pragma unroll
        for (int q = 0; q < (TRI == TRI_NONE ? 0 : MM::KPL / MM::CH); ++q) {
            TC af[WTM][MM::CH], bf[WTN][MM::CH];
            const int kk = h * MM::KPL + q * MM::CH;
#pragma unroll
            for (int i = 0; i < WTM; ++i) {
                const int rr = wm * WROWS + i * T + r;
                if (AKM) {
#pragma unroll
                    for (int e = 0; e < MM::CH; ++e) af[i][e] = as[(kk + e) * MM::PITCH_KM + rr];
                } else {
                    const u32x4 v = *(const ASTERIA_LDS u32x4 *)(as + rr * MM::PITCH_KC + kk);
                    *reinterpret_cast<u32x4 *>(&af[i][0]) = v;
                }
            }
#pragma unroll
            for (int j = 0; j < WTN; ++j) {
                const int cc = wn * WCOLS + j * T + r;
                if (BKM) {
#pragma unroll
                    for (int e = 0; e < MM::CH; ++e) bf[j][e] = bs[(kk + e) * MM::PITCH_KM + cc];
                } else {
                    const u32x4 v = *(const ASTERIA_LDS u32x4 *)(bs + cc * MM::PITCH_KC + kk);
                    *reinterpret_cast<u32x4 *>(&bf[j][0]) = v;
                }
            }
#pragma unroll
            for (int e = 0; e < MM::CH; ++e)
#pragma unroll
                for (int i = 0; i < WTM; ++i)
#pragma unroll
                    for (int j = 0; j < WTN; ++j)
                        if (TRI == TRI_ALL || j - i <= TRI) acc[i][j] = MM::mma(af[i][e], bf[j][e], acc[i][j]);
        }
    };
    if constexpr (!GUARD && MM::PREFETCH == 2) {
        // two register sets: slab j waits in set j % 2 from its global load, issued two iterations
        // ahead, until it is stored to LDS stage j % 2 at the end of iteration j - 1
        StA sa[2];
        StB sb[2];
        auto load = [&](auto set, int slab) {
            sa[decltype(set)::value].template load<false>(Ab, lda, row0, rowsA, slab * BK, BK, vecA, tid);
            sb[decltype(set)::value].template load<false>(Bb, ldb, col0, rowsB, slab * BK, BK, vecB, tid);
        };
        auto store = [&](auto set) {
            sa[decltype(set)::value].store(smem + decltype(set)::value * StA::LDS_ELEMS, tid);
            sb[decltype(set)::value].store(smemB + decltype(set)::value * StB::LDS_ELEMS, tid);
        };
        using S0 = std::integral_constant<int, 0>;
        using S1 = std::integral_constant<int, 1>;
        load(S0{}, 0);
        store(S0{});
        if (nk > 1) load(S1{}, 1);
        __syncthreads();
        for (int kt = 0; kt < nk; kt += 2) {
            if (kt + 2 < nk) load(S0{}, kt + 2);
            compute(0);
            if (kt + 1 < nk) store(S1{});
            __syncthreads();
            if (kt + 1 >= nk) break;
            if (kt + 3 < nk) load(S1{}, kt + 3);
            compute(1);
            if (kt + 2 < nk) store(S0{});
            __syncthreads();
        }
    } else {
        StA sa;
        StB sb;
        sa.template load<GUARD>(Ab, lda, row0, rowsA, 0, K, vecA, tid);
        sb.template load<GUARD>(Bb, ldb, col0, rowsB, 0, K, vecB, tid);
        sa.store(smem, tid);
        sb.store(smemB, tid);
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const int cur = kt & 1;
            if (kt + 1 < nk) {
                const int k0 = (kt + 1) * BK;
                sa.template load<GUARD>(Ab, lda, row0, rowsA, k0, K - k0, vecA, tid);
                sb.template load<GUARD>(Bb, ldb, col0, rowsB, k0, K - k0, vecB, tid);
            }
            compute(cur);
            if (kt + 1 < nk) {
                sa.store(smem + (cur ^ 1) * StA::LDS_ELEMS, tid);
                sb.store(smemB + (cur ^ 1) * StB::LDS_ELEMS, tid);
            }
            __syncthreads();
        }
    }
}

// Store one accumulated 128 x 128 tile: C = alpha acc + beta C, optional bf16 store, optional
// mirror (symmetric problems) and the root epilogue (T' = a I - g C and the residual partial sum).
// MM supplies the accumulator layout (tile edge T, NACC values per lane, acc_row) and the wave grid.
template <typename MM, typename TC>
__device__ __forceinline__ void gemm_epilogue(const GemmProblem &P, typename MM::acc_t (&acc)[MM::WTM][MM::WTN],
                                              int lt, int ti, int tj, int row0, int col0, int rowsA, int rowsB,
                                              int wm, int wn, int r, int h, int lane, int wave, int tid,
                                              float *red)
{
    constexpr int WTM = MM::WTM, WTN = MM::WTN;
    constexpr int WROWS = BM / MM::WAVES_M, WCOLS = BN / MM::WAVES_N;
    constexpr int T = MM::T;
    const int flags = P.flags;
    const int M = P.M, N = P.N;
    const bool sym = (flags & GEMM_SYM) != 0;
    const bool root = (flags & GEMM_EPI_ROOT) != 0;
    const TC alpha = (TC)P.alpha, beta = (TC)P.beta;
    // coefficients of T = a I - g C: per-problem device values (coef[0], coef[1]) or the table's
    const float *coef = root ? P.coef : nullptr;
    const TC ep_a = (TC)(coef ? coef[0] : P.ep_a), ep_g = (TC)(coef ? coef[1] : P.ep_g);
    void *C = P.C;
    TC *C2 = reinterpret_cast<TC *>(P.C2);
    const int ldc = P.ldc, ldc2 = P.ldc2;
    float rsum = 0.0f;
    // Fast fp32 stores need a full, aligned tile: in the 32 x 32 MFMA layout a lane owns 4
    // consecutive rows of one column, so the mirrored group C[col][row .. row + 3] is one aligned
    // 16-byte store (a scalar mirror store touches 64 different cache lines per instruction).
    const bool packed = (flags & GEMM_C_PACKED) != 0;
    bool handover = false;                      // fp64 compute only (a compile-time no for the fp32 kernels)
    if constexpr (sizeof(TC) == 8) handover = root && (flags & GEMM_EPI_HANDOVER) != 0;
    bool vec_c = false;
    if constexpr (sizeof(TC) == 4)
        vec_c = !packed && rowsA == BM && rowsB == BN && !(flags & (GEMM_C_BF16 | GEMM_EPI_HANDOVER)) && (ldc & 3) == 0 &&
                (reinterpret_cast<uintptr_t>(C) & 15u) == 0 &&
                (!root || (P.C3 == nullptr && (ldc2 & 3) == 0 && (reinterpret_cast<uintptr_t>(C2) & 15u) == 0));
#pragma unroll
    for (int i = 0; i < WTM; ++i) {
#pragma unroll
        for (int j = 0; j < WTN; ++j) {
            // one T x T MFMA block; all three cases below are uniform over the wavefront
            const int br = row0 + wm * WROWS + i * T, bc = col0 + wn * WCOLS + j * T;
            if (sym && br + T - 1 < bc) continue;           // entirely above the diagonal: mirrored from below
            const bool below = br >= bc + T;                // entirely below the diagonal
            const int col = bc + r;
            bool done = false;
            if constexpr (sizeof(TC) == 4) {
                if (vec_c && (flags & GEMM_STORE_T)) {
                    // a lane owns 4 consecutive rows of one column: one 16-byte store per group
                    ASTERIA_GLOBAL float *Cg = (ASTERIA_GLOBAL float *)C;
#pragma unroll
                    for (int g4 = 0; g4 < MM::NACC / 4; ++g4) {
                        const int rb = br + 8 * g4 + 4 * h;
                        floatx4 v4;
#pragma unroll
                        for (int e = 0; e < 4; ++e) v4[e] = alpha * acc[i][j][4 * g4 + e];
                        *(ASTERIA_GLOBAL floatx4 *)(Cg + (size_t)col * ldc + rb) = v4;
                    }
                    done = true;
                } else if (vec_c && (!sym || below)) {
                    ASTERIA_GLOBAL float *Cg = (ASTERIA_GLOBAL float *)C;
                    ASTERIA_GLOBAL float *C2g = (ASTERIA_GLOBAL float *)C2;
#pragma unroll
                    for (int g4 = 0; g4 < MM::NACC / 4; ++g4) {
                        const int rb = br + 8 * g4 + 4 * h;
                        floatx4 v4, t4;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float val = alpha * acc[i][j][4 * g4 + e];
                            if (beta != 0.0f) val += beta * Cg[(size_t)(rb + e) * ldc + col];
                            Cg[(size_t)(rb + e) * ldc + col] = val;
                            v4[e] = val;
                            if (root) {
                                const float d = (rb + e == col) ? 1.0f : 0.0f;
                                const float t2 = ep_a * d - ep_g * val;
                                C2g[(size_t)(rb + e) * ldc2 + col] = t2;
                                t4[e] = t2;
                                const float er = val - d;
                                rsum += sym ? 2.0f * er * er : er * er;
                            }
                        }
                        if (sym) {
                            *(ASTERIA_GLOBAL floatx4 *)(Cg + (size_t)col * ldc + rb) = v4;
                            if (root) *(ASTERIA_GLOBAL floatx4 *)(C2g + (size_t)col * ldc2 + rb) = t4;
                        }
                    }
                    done = true;
                }
            }
            if (done) continue;
            // Offsets of the block's element (br, bc) and of its transposed image (bc, br), and the row
            // pitch: dense row-major storage, or packed lower tiles - the whole MFMA block then lies in
            // one stored 128 x 128 tile, and a mirror image exists only inside a diagonal tile.
            size_t off_n = (size_t)br * ldc + bc, off_t = (size_t)bc * ldc + br;
            int ld_c = ldc;
            bool do_mirror = sym;
            if (packed) {
                off_n = packed_off(br, bc);
                ld_c = PACK_T;
                do_mirror = sym && br / PACK_T == bc / PACK_T;
                off_t = do_mirror ? packed_off(bc, br) : 0;
            }
#pragma unroll
            for (int v = 0; v < MM::NACC; ++v) {
                const int row = br + MM::acc_row(v, h);
                if (row >= M || col >= N) continue;
                if (sym && row < col) continue;   // the mirror of (col, row) covers it
                TC val = alpha * acc[i][j][v];
                const size_t at_n = off_n + (size_t)(row - br) * ld_c + (size_t)(col - bc);
                const size_t at_t = off_t + (size_t)(col - bc) * ld_c + (size_t)(row - br);
                const size_t at = (flags & GEMM_STORE_T) ? at_t : at_n;
                if (beta != (TC)0) val += beta * load_c<TC>(C, at, flags);
                if (!handover) {
                    store_c<TC>(C, at, val, flags);
                    if (do_mirror && row != col) store_c<TC>(C, at_t, val, flags);
                } else {
                    P.C4[(size_t)row * P.ldc4 + col] = (float)val;
                    if (sym && row != col) P.C4[(size_t)col * P.ldc4 + row] = (float)val;
                }
                if (root) {
                    const TC d = (row == col) ? (TC)1 : (TC)0;
                    const TC t2 = ep_a * d - ep_g * val;
                    if (!handover) {
                        C2[(size_t)row * ldc2 + col] = t2;
                        if (sym && row != col) C2[(size_t)col * ldc2 + row] = t2;
                    }
                    if (P.C3) {
                        P.C3[(size_t)row * P.ldc3 + col] = (float)t2;
                        if (sym && row != col) P.C3[(size_t)col * P.ldc3 + row] = (float)t2;
                    }
                    const float e = (float)(val - d);
                    rsum += (sym && row != col) ? 2.0f * e * e : e * e;
                }
            }
        }
    }
    if (root) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) rsum += __shfl_xor(rsum, off, 64);
        if (lane == 0) red[wave] = rsum;
        __syncthreads();
        if (tid == 0) {
            float t = 0.0f;
#pragma unroll
            for (int w = 0; w < MM::NTHR / 64; ++w) t += red[w];
            P.partial[lt] = t;
        }
    }
}

// In a diagonal tile of a symmetric product a wavefront multiplies only the blocks of its sub-tile
// that reach the diagonal or lie below it, so the positions of the wavefront grid carry unequal
// work.  Wavefronts w and w + 4 of a workgroup share a SIMD: with 8 wavefronts the positions are
// handed out so that each SIMD gets one of the four heaviest and, in reverse order, one of the four
// lightest.  role(w) is the grid position (wm WAVES_N + wn) wavefront w takes in such a tile.
template <class MM>
struct DiagRoles {
    static constexpr int NW = MM::WAVES_M * MM::WAVES_N;
    static constexpr int kept(int pos)
    {
        const int d = (pos / MM::WAVES_N) * MM::WTM - (pos % MM::WAVES_N) * MM::WTN;
        int c = 0;
        for (int i = 0; i < MM::WTM; ++i)
            for (int j = 0; j < MM::WTN; ++j)
                if (j - i <= d) ++c;
        return c;
    }
    static constexpr uint64_t packed()
    {
        int order[NW] = {};
        for (int w = 0; w < NW; ++w) order[w] = w;
        for (int a = 0; a < NW; ++a)              // stable selection sort, heaviest first
            for (int b = a + 1; b < NW; ++b)
                if (kept(order[b]) > kept(order[a])) {
                    const int t = order[b];
                    for (int c = b; c > a; --c) order[c] = order[c - 1];
                    order[a] = t;
                }
        uint64_t p = 0;
        for (int w = 0; w < NW; ++w) {
            int pos = w;
            if (NW == 8) pos = (w < 4) ? order[w] : order[NW - 1 - (w - 4)];
            p |= (uint64_t)pos << (4 * w);
        }
        return p;
    }
    static_assert(NW <= 16, "4 bits per wavefront");
    __device__ static __forceinline__ int role(int w)
    {
        constexpr uint64_t P = packed();
        return (int)((P >> (4 * w)) & 15u);
    }
};

// calls run(integral_constant<d>) for the value D in [LO, HI] equal to d; only values that a
// wavefront grid with steps SM, SN can produce (combinations i SM - j SN) get an instance
constexpr int tri_gcd(int a, int b) { return b == 0 ? a : tri_gcd(b, a % b); }
template <int D, int HI, int SM, int SN, class F>
__device__ __forceinline__ void tri_try(int d, bool &ran, F &run)
{
    if constexpr (D <= HI) {
        constexpr int G = tri_gcd(SM, SN);
        if constexpr ((D % G + G) % G == 0) {
            if (!ran && d == D) { run(std::integral_constant<int, D>{}); ran = true; }
        }
        tri_try<D + 1, HI, SM, SN>(d, ran, run);
    }
}

// ---- the kernel -------------------------------------------------------------------------------
template <typename TC, typename TA, typename TB, bool AKM, bool BKM>
__global__ __launch_bounds__(Mma<TC>::NTHR, Mma<TC>::MIN_WAVES) void gemm_grouped_kernel(const GemmProblem *__restrict__ probs,
                                                                int nprobs, int total_tiles,
                                                                const int *__restrict__ state)
{
    using MM = Mma<TC>;
    constexpr int BK = MM::BK;
    constexpr int WTM = MM::WTM, WTN = MM::WTN;
    constexpr int T = MM::T;

    extern __shared__ __align__(16) unsigned char smem_raw[];
    ASTERIA_LDS TC *smem = (ASTERIA_LDS TC *)smem_raw;
    __shared__ float red[MM::NTHR / 64];

    // XCD-aware order: workgroup b lands on XCD b % 8; give every XCD a contiguous tile range
    // so the tiles of one problem share that XCD's L2.
    const int per_xcd = (total_tiles + NUM_XCD - 1) / NUM_XCD;
    const int t_global = (int)(blockIdx.x % NUM_XCD) * per_xcd + (int)(blockIdx.x / NUM_XCD);
    if (t_global >= total_tiles) return;

    // binary search: last problem with tile_start <= t_global
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
    if (P.gate && *P.gate != 0) return;
    const int flags = P.flags;
    const int lt = t_global - P.tile_start;
    int ti, tj;
    if (flags & GEMM_SYM) tri_decode(lt, ti, tj);
    else { ti = lt / P.tiles_n; tj = lt % P.tiles_n; }

    const int M = P.M, N = P.N, K = P.K;
    const int row0 = ti * BM, col0 = tj * BN;
    const int rowsA = min(BM, M - row0);
    const int rowsB = min(BN, N - col0);
    const TA *Ab = reinterpret_cast<const TA *>(P.A);
    const TB *Bb = reinterpret_cast<const TB *>(P.B);
    const int lda = P.lda, ldb = P.ldb;
    const bool vecA = ((reinterpret_cast<uintptr_t>(Ab) & 15u) == 0) && ((((size_t)lda * sizeof(TA)) & 15u) == 0);
    const bool vecB = ((reinterpret_cast<uintptr_t>(Bb) & 15u) == 0) && ((((size_t)ldb * sizeof(TB)) & 15u) == 0);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    // position of the wavefront's sub-tile in the wavefront grid; diagonal tiles of symmetric
    // products hand the positions out in another order (see DiagRoles)
    int role = __builtin_amdgcn_readfirstlane(wave);
    const bool diag_tri = !AKM && !BKM && (flags & GEMM_SYM) && ti == tj;
    if (diag_tri) role = DiagRoles<MM>::role(role);
    const int wm = role / MM::WAVES_N, wn = role % MM::WAVES_N;
    const int r = lane % T;   // row (A) / column (B) inside an MFMA tile
    const int h = lane / T;   // k group

    typename MM::acc_t acc[WTM][WTN];
#pragma unroll
    for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j)
#pragma unroll
            for (int v = 0; v < MM::NACC; ++v) acc[i][j][v] = (TC)0;

    // Fast path: full tile, whole slabs, aligned vectors -> no per-element guards in the loop.
    const bool fast = vecA && vecB && rowsA == BM && rowsB == BN && (K % BK) == 0;
    // diagonal tile of a symmetric product: only the blocks on and below the diagonal are stored,
    // so only those are multiplied (the choice is uniform over a wavefront)
    auto run = [&](auto tri) {
        gemm_mainloop<TC, TA, TB, AKM, BKM, false, decltype(tri)::value>(acc, Ab, Bb, lda, ldb, row0, col0, rowsA, rowsB,
                                                                        K, vecA, vecB, smem, tid, wm, wn, r, h);
    };
    if (fast) {
        constexpr int SM = BM / MM::WAVES_M / T, SN = BN / MM::WAVES_N / T;   // blocks per wavefront step
        bool ran = false;
        if constexpr (!AKM && !BKM) {
            if (diag_tri) {
                const int d = wm * SM - wn * SN;
                if (d < -(WTM - 1)) { run(std::integral_constant<int, TRI_NONE>{}); ran = true; }
                else if (d <= WTN - 2) {
                    // the partial patterns this wavefront grid can produce, one loop instance each
                    tri_try<-(WTM - 1), WTN - 2, SM, SN>(d, ran, run);
                }
            }
        }
        if (!ran) run(std::integral_constant<int, TRI_ALL>{});
    }
    else
        gemm_mainloop<TC, TA, TB, AKM, BKM, true>(acc, Ab, Bb, lda, ldb, row0, col0, rowsA, rowsB, K, vecA, vecB,
                                                  smem, tid, wm, wn, r, h);

    gemm_epilogue<MM, TC>(P, acc, lt, ti, tj, row0, col0, rowsA, rowsB, wm, wn, r, h, lane, wave, tid, red);
}

template <typename TC, typename TA, typename TB, bool AKM, bool BKM>
constexpr size_t gemm_lds_bytes()
{
    return sizeof(TC) * 2 * (size_t)(OperandStage<TC, TA, AKM>::LDS_ELEMS + OperandStage<TC, TB, BKM>::LDS_ELEMS);
}

// Enqueue one grouped launch.  probs / state are device pointers (state may be null when no
// problem refers to it).
template <typename TC, typename TA, typename TB, bool AKM, bool BKM>
inline hipError_t launch_gemm_grouped(const GemmProblem *probs, int nprobs, int total_tiles,
                                      const int *state, hipStream_t stream)
{
    if (total_tiles <= 0 || nprobs <= 0) return hipSuccess;
    auto kern = gemm_grouped_kernel<TC, TA, TB, AKM, BKM>;
    constexpr size_t lds = gemm_lds_bytes<TC, TA, TB, AKM, BKM>();
    static bool configured[MAX_DEVICES] = {};
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds, configured); e != hipSuccess) return e;
    const int per_xcd = (total_tiles + NUM_XCD - 1) / NUM_XCD;
    constexpr int kind = (sizeof(TC) == 8 ? 1 : 0) | (sizeof(TA) == 2 ? 2 : 0) | (sizeof(TB) == 2 ? 4 : 0) |
                         (AKM ? 8 : 0) | (BKM ? 16 : 0);
    profile_begin(kind, stream);
    hipLaunchKernelGGL(kern, dim3(per_xcd * NUM_XCD), dim3(Mma<TC>::NTHR), lds, stream, probs, nprobs,
                       total_tiles, state);
    profile_end(stream);
    return hipGetLastError();
}

inline int tri_tiles(int n)
{
    const int t = (n + BM - 1) / BM;
    return t * (t + 1) / 2;
}

}  // namespace asteria
