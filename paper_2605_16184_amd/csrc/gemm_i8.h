// gemm_i8.h - products of symmetric fp64 matrices on the int8 matrix cores.
//
// An fp64 operand S is written as  S = diag(S) + O  and the off-diagonal part O row by row as
//     O[i][k] = 2^e_i * sum_{s < NS} d_s[i][k] 2^(-6 - 7 s),   d_s integers with |d_s| <= 64,
// e_i = exponent of the largest |O[i][k]| of the row (so |O[i][k]| 2^-e_i < 1): NS slices of 7 bits
// below a per-row exponent, 7 NS + 1 bits in all.  The product of two such operands is
//     (Sa Sb)[i][j] = 2^(e_i + f_j) sum_l 2^(-12 - 7 l) sum_{s + t = l} sum_k d_s[i][k] d'_t[j][k]
//                     + diag_a[i] Sb[i][j] + Sa[i][j] diag_b[j]            (i != j; B symmetric)
// and diag_a[i] diag_b[i] in place of the last two terms for i = j.  The integer sums are exact in the
// int32 accumulators of v_mfma_i32_32x32x32_i8 (|sum| <= NS K 2^12 < 2^31 for K <= 100000); the levels
// l = s + t < NS are kept, the dropped ones are of relative size 2^(-7 NS) of the row scales.
// Holding the diagonal out matters: a matrix a I - g M has a diagonal far above its off-diagonal
// entries, and with it inside the slices the dropped levels would be measured against the diagonal.
//
// Slice layout in memory ("planes"): row i, block b of 32 consecutive k, slice s, 32 bytes:
//     planes[i * row_bytes + (b * NS + s) * 32 + k % 32],   kb = ceil(n / 32), row_bytes >= kb NS 32,
// rows padded with zero rows to a multiple of 128 and k padded with zeros to a multiple of 32, so
// the product kernel reads whole tiles without guards.
//
// B mode 1: the B operand of the product is M, and the planes in buffer `bbuf` are those of
// T = a I - g M (already cut for T T): off-diagonal M = -(off-diagonal T) / g, so the integer sums
// are scaled by bscale = -1 / g and the diagonal of M is read from the matrix itself.  M is then
// never cut into slices.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm.h"

namespace asteria {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef double doublex16 __attribute__((ext_vector_type(16)));
typedef double doublex2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Per factor: two sliced operand buffers (0: the A operand of every product, 1: the B operand where
// it is another matrix) and the decision where the current product runs.
struct I8Factor {
    int8_t *planes[2];
    int *expo[2];        // per row (padded): e_i
    double *diag[2];     // per row (padded): S[i][i]
    unsigned rmax[2];    // float bits: largest off-diagonal |entry| of the operand
    unsigned dmax[2];    // float bits: largest |diagonal entry|
    int gate;            // number of slices the current product is computed with on the int8 cores, or 0: fp64 cores
    int n, kb;
    float bscale;        // see the B modes of the product kernel
};

inline size_t i8_rows(int n) { return (size_t)((n + 127) & ~127); }
// Bytes between the slice rows of consecutive matrix rows: the kb blocks, padded to an odd multiple
// of 128 bytes - with a power-of-two stride the 128 rows a tile loads side by side fall on the same
// L2 / memory channels.
__host__ __device__ inline size_t i8_row_bytes(int kb, int ns)
{
    const size_t units = ((size_t)kb * 32u * (size_t)ns + 127) / 128;
    return (units | 1) * 128;
}
inline size_t i8_plane_bytes(int n, int ns) { return i8_rows(n) * i8_row_bytes((n + 31) / 32, ns); }

// ---- slicing ------------------------------------------------------------------------------------
// One wavefront per row (rows of up to 2048 entries are parked in LDS between finding the row scale
// and cutting, longer ones are read twice).  Grid: x = groups of 4 rows (of the largest factor, padded), y = problem.
// Reads operand A (use_b = 0) or B (use_b = 1) of the problem as an n x n fp64 matrix with an even
// leading dimension and a 16-byte aligned base, writes buffer `buf` of the factor.
constexpr int I8_SLICE_LDS_K = 2048;   // longest (padded) row the slicing kernel parks in LDS (4 rows per workgroup: 70 KB)
template <int NS>
__global__ __launch_bounds__(256) void i8_slice_kernel(const GemmProblem *__restrict__ probs, I8Factor *__restrict__ xf,
                                                       const int *__restrict__ state, int use_b, int buf, int lds_k)
{
    const GemmProblem &P = probs[blockIdx.y];
    if (P.state_idx >= 0) {
        const int st = state[P.state_idx];
        if (!((1 << st) & P.state_mask)) return;
    }
    extern __shared__ __align__(16) double slice_lds[];   // 4 rows of ceil(lds_k / 16) * 17 doubles, or nothing
    I8Factor &X = xf[P.state_idx];
    const int n = P.M;
    const int npad = (n + 127) & ~127;
    const int lane = threadIdx.x & 63;
    const int row = (int)blockIdx.x * 4 + (int)(threadIdx.x >> 6);
    if (row >= npad) return;
    const int kb = X.kb;
    const size_t rowbytes = i8_row_bytes(kb, NS);
    int8_t *dst = X.planes[buf] + (size_t)row * rowbytes;
    if (row >= n) {
        for (size_t o = (size_t)lane * 16; o < rowbytes; o += 64 * 16)
            *(ASTERIA_GLOBAL u32x4 *)(dst + o) = (u32x4){0u, 0u, 0u, 0u};
        if (lane == 0) { X.expo[buf][row] = 0; X.diag[buf][row] = 0.0; }
        return;
    }
    const double *S = reinterpret_cast<const double *>(use_b ? P.B : P.A);
    const int ld = use_b ? P.ldb : P.lda;
    const double *src = S + (size_t)row * ld;
    const int kend = kb * 32;
    auto finish_scale = [&](double mx, double dg) -> int {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            mx = fmax(mx, __shfl_xor(mx, off, 64));
            dg += __shfl_xor(dg, off, 64);      // one lane holds the diagonal, the others 0
        }
        int e = 0;
        if (mx > 0.0 && mx < 1e300) (void)frexp(mx, &e);   // mx = m 2^e, 0.5 <= m < 1
        if (lane == 0) {
            X.expo[buf][row] = e;
            X.diag[buf][row] = dg;
            atomicMax(&X.rmax[buf], __float_as_uint(fminf((float)mx * 1.0000002f, 3.0e38f)));
            atomicMax(&X.dmax[buf], __float_as_uint(fminf((float)fabs(dg), 3.0e38f)));
        }
        return e;
    };
    // 8 values (diagonal and padding already zeroed) -> NS x 8 bytes at d, d + 32, ...
    auto cut8 = [&](double (&u)[8], int e, int8_t *d) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            double t = ldexp(u[j], 6 - e);      // |t| < 64
            if (!(fabs(t) <= 64.0)) t = 0.0;    // non-finite input: the caller's state machine reports it
            u[j] = t;
        }
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            uint32_t w0 = 0u, w1 = 0u;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const double q = rint(u[j]);
                u[j] = (u[j] - q) * 128.0;      // exact: the remainder has at most 46 bits left
                const uint32_t b = (uint32_t)((int)q & 0xff);
                if (j < 4) w0 |= b << (8 * j); else w1 |= b << (8 * (j - 4));
            }
            *(ASTERIA_GLOBAL u32x2 *)(d + s * 32) = (u32x2){w0, w1};
        }
    };
    if (kend <= lds_k) {
        // One read of the matrix: coalesced loads (2 consecutive k per lane), the row parked in the
        // wavefront's LDS buffer, then 16 consecutive k per lane from there (16-byte stores).  Chunks
        // of 16 doubles are 17 doubles apart, which spreads the lanes' chunk reads over the banks.
        ASTERIA_LDS double *rowbuf = (ASTERIA_LDS double *)slice_lds + (threadIdx.x >> 6) * (lds_k / 16 * 17);
        double mx = 0.0, dg = 0.0;
#pragma unroll 4
        for (int k0 = lane * 2; k0 < kend; k0 += 128) {
            doublex2_t v = {0.0, 0.0};
            if (k0 < n) v = *(const ASTERIA_GLOBAL doublex2_t *)(src + k0);
            double v0 = v[0], v1 = (k0 + 1 < n) ? v[1] : 0.0;
            if (k0 == row) { dg = v0; v0 = 0.0; }
            if (k0 + 1 == row) { dg = v1; v1 = 0.0; }
            mx = fmax(mx, fmax(fabs(v0), fabs(v1)));
            ASTERIA_LDS double *w = rowbuf + (k0 >> 4) * 17 + (k0 & 15);
            w[0] = v0; w[1] = v1;
        }
        const int e = finish_scale(mx, dg);
        __builtin_amdgcn_s_waitcnt(0xc07f);      // lgkmcnt(0): the wavefront's LDS writes have landed
        for (int k0 = lane * 16; k0 < kend; k0 += 1024) {
            double u[16];
            const ASTERIA_LDS double *rd = rowbuf + (k0 >> 4) * 17;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                double t = ldexp(rd[j], 6 - e);      // |t| < 64
                if (!(fabs(t) <= 64.0)) t = 0.0;
                u[j] = t;
            }
            int8_t *d = dst + (size_t)(k0 >> 5) * (32 * NS) + (k0 & 31);
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                u32x4 w = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const double q = rint(u[j]);
                    u[j] = (u[j] - q) * 128.0;
                    w[j >> 2] |= (uint32_t)((int)q & 0xff) << (8 * (j & 3));
                }
                *(ASTERIA_GLOBAL u32x4 *)(d + s * 32) = w;
            }
        }
        return;
    }
    // longer rows: pass 1 finds the scale, pass 2 reads the row again
    double mx = 0.0, dg = 0.0;
    for (int k0 = lane * 2; k0 < n; k0 += 128) {
        const doublex2_t v = *(const ASTERIA_GLOBAL doublex2_t *)(src + k0);
        const double v0 = v[0], v1 = (k0 + 1 < n) ? v[1] : 0.0;
        if (k0 == row) dg = v0; else mx = fmax(mx, fabs(v0));
        if (k0 + 1 == row) dg = v1; else mx = fmax(mx, fabs(v1));
    }
    const int e = finish_scale(mx, dg);
    for (int k0 = lane * 8; k0 < kend; k0 += 512) {
        double u[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k = k0 + 2 * j;
            doublex2_t v = {0.0, 0.0};
            if (k < n) v = *(const ASTERIA_GLOBAL doublex2_t *)(src + k);
            u[2 * j] = (k == row) ? 0.0 : v[0];
            u[2 * j + 1] = (k + 1 >= n || k + 1 == row) ? 0.0 : v[1];
        }
        cut8(u, e, dst + (size_t)(k0 >> 5) * (32 * NS) + (k0 & 31));
    }
}

// lds_k and the dynamic LDS size of a slicing launch whose longest row has n_max entries
inline int i8_slice_lds_k(int n_max) { const int k = (n_max + 31) & ~31; return k <= I8_SLICE_LDS_K ? k : 0; }
inline size_t i8_slice_lds_bytes(int lds_k) { return (size_t)4 * ((lds_k + 15) / 16 * 17) * sizeof(double); }

// ---- where a product runs ------------------------------------------------------------------------
// The dropped levels s + t >= NS contribute, per entry, about 0.33 sqrt(K (NS - 1)) 2^(-7 NS) ra rb
// (ra, rb: the row scales, bounded by the largest off-diagonal entries), measured here against
// theta * lo * da * db: lo = the bottom of the spectrum of the current M (an error of relative size u
// in the chain products costs about u / lo in the root), da db = the product of the largest diagonal
// entries as a lower bound of ||Sa|| ||Sb||.  One thread per factor; clears the maxima for the next
// operand.
// theta for a prefix of two fp64 iterations (six products); a longer prefix shares the same total: the
// host passes theta * 2 / (number of fp64 iterations)
constexpr float I8_THETA = 2e-5f;

// `scal` points at the factor's (lo, hi, g) of the current iteration: the interval that holds the
// spectrum of the current M and the g of the current T = a I - g M.
__global__ void i8_gate_kernel(I8Factor *__restrict__ xf, int nf, const float *__restrict__ scal, int scal_stride_bytes,
                               int ns_min, int ns_max, int abuf, int bbuf, int bmode, float theta,
                               const int *__restrict__ state, double *counters)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nf) return;
    I8Factor &X = xf[i];
    const float *sc = reinterpret_cast<const float *>(reinterpret_cast<const char *>(scal) + (size_t)i * scal_stride_bytes);
    const float lo = sc[0], hi = sc[1], g = sc[2];
    const float ra = __uint_as_float(X.rmax[abuf]), da = __uint_as_float(X.dmax[abuf]);
    float rb = __uint_as_float(X.rmax[bbuf]), db = __uint_as_float(X.dmax[bbuf]);
    if (bmode == 1) {
        // B = M seen through the planes of T: off-diagonal scale / g, and ||M|| is the top of its interval
        rb = (g > 0.0f) ? rb / g : 3.0e38f;
        db = hi;
        X.bscale = (g > 0.0f) ? -1.0f / g : 0.0f;
    }
    const float allowed = theta * lo * da * db;
    int gsel = 0;
    for (int ns = ns_max; ns >= ns_min; --ns) {       // the fewest slices that pass
        const float est = 0.33f * sqrtf((float)X.n * (float)(ns - 1)) * exp2f(-7.0f * (float)ns) * ra * rb;
        if (est <= allowed && allowed > 0.0f) gsel = ns;
    }
    X.gate = gsel;
    if (counters && state[i] == 0)      // measurement aid: where the running factors' products go
        atomicAdd(&counters[gsel == 0 ? 0 : gsel - 3], (double)X.n * (double)X.n * (double)(X.n + 1));
    // buffer 0 is cut anew before every product; buffer 1 holds T from the first product of an
    // iteration to the last (B mode 1)
    X.rmax[0] = 0u; X.dmax[0] = 0u;
    if (bmode == 1) { X.rmax[1] = 0u; X.dmax[1] = 0u; }
}

// ---- the product kernel --------------------------------------------------------------------------
// A workgroup of 4 wavefronts (2 x 2, 64 x 32 each: two 32 x 32 MFMA tiles) computes one half
// (128 rows x 64 columns) of a 128 x 128 lower-triangle tile, so that a CU holds two workgroups
// and the epilogue of one (fp64 assembly, 16 + 16..40 bytes of HBM traffic per element) runs under
// the K loop of the other.  One slab = one block of 32 k for all NS slices, double-buffered in LDS
// as [slice][k half][row][16 bytes], so the 32 lanes of one k half read 512 contiguous bytes per
// fragment; each [slice][k half] piece is padded by 16 bytes, which spreads the 2 NS pieces of one
// row, which consecutive lanes store, over different banks.  Per slab a wavefront reads 3 NS
// fragments and issues NS (NS + 1) MFMAs into NS level accumulators per MFMA tile.  NSL is the
// number of slices the planes were written with: a product may use only the leading NS of them
// (the slices are digits, most significant first).
struct MmaI8 {
    static constexpr int T = 32;
    static constexpr int NACC = 16;
    // the common epilogue places a wavefront at (wm * 128 / WAVES_M, wn * 128 / WAVES_N): 64-row and
    // 32-column steps; the column origin it is given is that of the half tile
    static constexpr int WAVES_M = 2, WAVES_N = 4;
    static constexpr int NTHR = 256;
    static constexpr int WTM = 2, WTN = 1;
    typedef doublex16 acc_t;
    __device__ static __forceinline__ int acc_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }
};
constexpr int I8_TN = 64;        // columns per workgroup

// one half tile with NS of the NSL slices the planes hold; lt = tile within the problem, half = 0 | 1
template <int NS, int NSL>
__device__ __forceinline__ void i8_tile(const GemmProblem &P, const I8Factor &X, int lt, int half, int abuf, int bbuf,
                                        int bmode, unsigned char *smem_raw, float *red)
{
    constexpr int PIECE_A = 128 * 16 + 16;           // one k half of one slice: rows x 16 bytes, padded
    constexpr int PIECE_B = I8_TN * 16 + 16;
    constexpr int OPERAND_A = 2 * NS * PIECE_A;
    constexpr int STAGE = OPERAND_A + 2 * NS * PIECE_B;
    constexpr int CPR = 2 * NS;                      // 16-byte chunks per row and slab
    constexpr int CHUNKS_A = 128 * CPR;
    constexpr int TOTAL = (128 + I8_TN) * CPR;
    constexpr int NV = (TOTAL + 255) / 256;

    ASTERIA_LDS unsigned char *smem_i8 = (ASTERIA_LDS unsigned char *)smem_raw;
    int ti, tj;
    tri_decode(lt, ti, tj);                          // symmetric products only
    const int n = P.M;
    const int row0 = ti * BM, col0 = tj * BN + half * I8_TN;
    const int kb = X.kb;
    const size_t rowbytes = i8_row_bytes(kb, NSL);
    const int8_t *Ap = X.planes[abuf] + (size_t)row0 * rowbytes;
    const int8_t *Bp = X.planes[bbuf] + (size_t)col0 * rowbytes;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 31, h = lane >> 5;

    // staging: chunk idx = tid + 256 v over both operands
    const int8_t *gsrc[NV];
    int ldst[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int idx = min(tid + 256 * v, TOTAL - 1);
        const bool isb = idx >= CHUNKS_A;
        const int c = isb ? idx - CHUNKS_A : idx;
        const int row = c / CPR, piece = c % CPR;
        gsrc[v] = (isb ? Bp : Ap) + (size_t)row * rowbytes + piece * 16;
        ldst[v] = isb ? OPERAND_A + piece * PIECE_B + row * 16 : piece * PIECE_A + row * 16;
    }
    // Register sets for slabs in flight from global memory.  Two (NS <= 4, where the budget allows)
    // give a load two slabs of MFMA work to arrive: a third of the requests miss L2.  The loads of
    // the deeper pipeline are unconditional (the slab index is clamped), so that the count of
    // loads issued after the set being stored is known statically and the wait before the store
    // leaves the younger set in flight.
    constexpr int DEPTH = NS <= 4 ? 2 : 1;
    u32x4 stg[DEPTH][NV];
    auto gload = [&](u32x4 (&set)[NV], int slab) {
#pragma unroll
        for (int v = 0; v < NV; ++v)
            if (TOTAL % 256 == 0 || tid + 256 * v < TOTAL)
                set[v] = *(const ASTERIA_GLOBAL u32x4 *)(gsrc[v] + (size_t)slab * (32 * NSL));
    };
    auto lstore = [&](const u32x4 (&set)[NV], int buf) {
#pragma unroll
        for (int v = 0; v < NV; ++v)
            if (TOTAL % 256 == 0 || tid + 256 * v < TOTAL)
                *(ASTERIA_LDS u32x4 *)(smem_i8 + buf * STAGE + ldst[v]) = set[v];
    };

    i32x16 acc[NS][2];
#pragma unroll
    for (int l = 0; l < NS; ++l)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[l][i][v] = 0;

    auto compute = [&](int cur) {
        const ASTERIA_LDS unsigned char *LA = smem_i8 + cur * STAGE;
        const ASTERIA_LDS unsigned char *LB = LA + OPERAND_A;
        i32x4 a[NS][2], b[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
                a[s][i] = *(const ASTERIA_LDS i32x4 *)(LA + (2 * s + h) * PIECE_A + (wm * 64 + i * 32 + r) * 16);
            b[s] = *(const ASTERIA_LDS i32x4 *)(LB + (2 * s + h) * PIECE_B + (wn * 32 + r) * 16);
        }
        // consecutive MFMAs write different accumulators
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int t = 0; t < NS - s; ++t)
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    acc[s + t][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[s][i], b[t], acc[s + t][i], 0, 0, 0);
    };

    gload(stg[0], 0);
    lstore(stg[0], 0);
    if constexpr (DEPTH == 1) {
        __syncthreads();
        int cur = 0;
        for (int slab = 0; slab < kb; ++slab) {
            const bool more = slab + 1 < kb;
            if (more) gload(stg[0], slab + 1);
            compute(cur);
            if (more) lstore(stg[0], cur ^ 1);
            __syncthreads();
            cur ^= 1;
        }
    } else {
        // set 0 carries the odd slabs, set 1 the even ones; slabs are taken in pairs
        const int last = kb - 1;
        gload(stg[0], min(1, last));
        __syncthreads();
        for (int slab = 0; slab < kb; slab += 2) {
            gload(stg[DEPTH - 1], min(slab + 2, last));
            compute(0);
            lstore(stg[0], 1);                         // slab + 1 (a copy of the last slab if there is none)
            __syncthreads();
            gload(stg[0], min(slab + 3, last));
            if (slab + 1 < kb) compute(1);
            lstore(stg[DEPTH - 1], 0);                 // slab + 2
            __syncthreads();
        }
    }

    // levels -> fp64, row and column scales, the held-out diagonals
    const int *ea = X.expo[abuf], *eb = X.expo[bbuf];
    const double *da = X.diag[abuf], *db = X.diag[bbuf];
    const double *Sa = reinterpret_cast<const double *>(P.A), *Sb = reinterpret_cast<const double *>(P.B);
    const int lda = P.lda, ldb = P.ldb;
    doublex16 accd[2][1];
    const int col = col0 + wn * 32 + r;
    const bool col_ok = col < n;
    const int ecol = eb[col];                  // the arrays are padded to whole tiles
    const bool same = bmode == 0 && P.A == P.B && abuf == bbuf;
    const double bs = bmode == 1 ? (double)X.bscale : 1.0;
    const double dcol = bmode == 1 ? (col_ok ? Sb[(size_t)col * ldb + col] : 0.0) : db[col];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = row0 + wm * 64 + i * 32 + MmaI8::acc_row(v, h);
            double s = 0.0;
#pragma unroll
            for (int l = NS - 1; l >= 0; --l) s += (double)acc[l][i][v] * (1.0 / (double)(1ull << (12 + 7 * l)));
            double val = 0.0;
            if (col_ok && row < n) {
                val = ldexp(s, ea[row] + ecol) * bs;
                const double drow = da[row];
                if (row == col) val += drow * dcol;
                else if (same) val += Sa[(size_t)row * lda + col] * (drow + dcol);     // a square: one load
                else val += drow * Sb[(size_t)row * ldb + col] + Sa[(size_t)row * lda + col] * dcol;
            }
            accd[i][0][v] = val;
        }
    }
    const int rowsA = min(BM, n - row0), rowsB = min(I8_TN, n - col0);
    // the residual partial sums of the two halves of a tile go to separate slots
    const int tpr = (n + BM - 1) / BM;
    const int slot = lt + half * (tpr * (tpr + 1) / 2);
    gemm_epilogue<MmaI8, double>(P, accd, slot, ti, tj, row0, col0, rowsA, rowsB, wm, wn, r, h, lane, wave, tid, red);
}

// One launch serves every slice count the planes allow: the factor's gate picks the tile routine
// (a launch per count would add a grid of workgroups that only look up their factor and leave).
// Two consecutive workgroups share a 128 x 128 tile (and with it the A rows in L2).
template <int NSL>
__global__ __launch_bounds__(256, 2) void gemm_i8_grouped_kernel(const GemmProblem *__restrict__ probs,
                                                                 const I8Factor *__restrict__ xf, int nprobs,
                                                                 int total_tiles, const int *__restrict__ state, int abuf,
                                                                 int bbuf, int bmode)
{
    extern __shared__ __align__(16) unsigned char smem_i8_raw[];
    __shared__ float red[4];

    const int total_wg = 2 * total_tiles;
    const int per_xcd = (total_wg + NUM_XCD - 1) / NUM_XCD;
    const int w_global = (int)(blockIdx.x % NUM_XCD) * per_xcd + (int)(blockIdx.x / NUM_XCD);
    if (w_global >= total_wg) return;
    const int t_global = w_global >> 1, half = w_global & 1;
    int lo = 0, hi = nprobs - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (probs[mid].tile_start <= t_global) lo = mid; else hi = mid - 1;
    }
    const GemmProblem &P = probs[lo];
    {
        const int st = state[P.state_idx];
        if (!((1 << st) & P.state_mask)) return;
    }
    const I8Factor &X = xf[P.state_idx];
    const int g = X.gate;
    const int lt = t_global - P.tile_start;
    if (g == 4) i8_tile<4, NSL>(P, X, lt, half, abuf, bbuf, bmode, smem_i8_raw, red);
    if constexpr (NSL >= 5) {
        if (g == 5) i8_tile<5, NSL>(P, X, lt, half, abuf, bbuf, bmode, smem_i8_raw, red);
    }
}

template <int NSL>
hipError_t launch_gemm_i8_grouped(const GemmProblem *d_probs, const I8Factor *d_xf, int nprobs, int total_tiles,
                                  const int *d_state, int abuf, int bbuf, int bmode, hipStream_t stream)
{
    if (nprobs <= 0 || total_tiles <= 0) return hipSuccess;
    constexpr int LDS_BYTES = 2 * 2 * NSL * ((128 * 16 + 16) + (I8_TN * 16 + 16));
    static bool configured[MAX_DEVICES] = {};
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(gemm_i8_grouped_kernel<NSL>), LDS_BYTES, configured);
        e != hipSuccess) return e;
    const int per_xcd = (2 * total_tiles + NUM_XCD - 1) / NUM_XCD;
    profile_begin(300 + NSL, stream);
    hipLaunchKernelGGL(gemm_i8_grouped_kernel<NSL>, dim3(per_xcd * NUM_XCD), dim3(256), LDS_BYTES, stream, d_probs, d_xf,
                       nprobs, total_tiles, d_state, abuf, bbuf, bmode);
    profile_end(stream);
    return hipGetLastError();
}

}  // namespace asteria
