// asteria_inverse_root: X = ((A + A^T)/2 + eps I)^(-1/p) for a batch of symmetric factors
// (the inverse roots of paper Eq. 1; the O(d^3) update of paper Sec. I / III-B), computed
// entirely on the device:
//
//   1. lambda_max(A) by a Lanczos process (HBM-streaming mat-vec, wavefront reductions, the small
//      tridiagonal eigenproblem per factor on the device, per-factor early stop).
//   2. Scaling  s = 1 / ((1 + margin) lambda_max + eps),  M_0 = s (A + eps I),  X_0 = s^(1/p) I,
//      so the spectrum of M_0 lies in (0, 1].
//   3. Coupled iteration  T = a I - g M,  X <- X T,  M <- T^p M  (coefficients a, g adapted per
//      factor and iteration to the interval that holds M's spectrum, or the classical Newton
//      values a = (p + 1) / p, g = 1 / p).  Every product is one symmetric grouped GEMM on the
//      matrix cores; the epilogue of the M-update also emits the next T and the per-tile partial
//      sums of ||M - I||_F^2.  A per-factor state machine on the device (running -> last X
//      update -> done) lets finished factors drop out without any host round trip: their
//      workgroups exit at once.
//   4. The leading iterations of the M-chain keep fp64 matrices, where the smallest eigenvalues
//      of M are still comparable to fp32 round-off.  Their products run on the int8 matrix cores:
//      each operand is cut into its diagonal and 7-bit integer slices under a per-row exponent,
//      the integer sums are exact and the result is assembled in fp64 (gemm_i8.h); per factor
//      and product a device-side estimate of what the dropped slice pairs cost picks 4 or 5
//      slices or sends the product to the fp64 matrix cores.  The state is then cast to fp32 and
//      continues on
//      the fp16 matrix cores with every fp32 operand split into two fp16 terms (2^-22 per
//      operand; the fp32 matrix cores serve pinned options, absolute eps and very large n).  X
//      is kept in fp32 throughout and its updates run on the fp16 cores from the start.
//
// Per iteration: 1 control kernel + up to 4 launches (X T; T T; T^2 T^2; T^4 M); in the fp64
// iterations each chain product is a slicing pass, a decision kernel, the int8 launch and the
// fp64 launch for the factors the decision kept there.
#include <math.h>
#include <stddef.h>

#include <algorithm>
#include <vector>

#include "common.h"
#include "gemm.h"
#include "gemm_bf16.h"
#include "gemm_i8.h"
#include "root_schedule.h"

using namespace asteria;

namespace {

constexpr int PM_ROWS = 32;   // rows of A per mat-vec workgroup (8 per wavefront)
constexpr int LZ_MAX = 128;   // most Lanczos steps of the lambda_max estimate (size of the recurrence kept per factor)

enum : int { ST_RUN = 0, ST_LAST = 1, ST_DONE = 2, ST_FAIL = 3 };

// spectrum of M within 1 +- ROOT_STOP_DEV: one more X update finishes the factor
constexpr float ROOT_STOP_DEV = 1e-2f;
// accepted truncation error of the result per eigen-direction (a third of the 2e-3 accuracy bar
// on the relative Frobenius error, which averages over directions)
constexpr float ROOT_X_TOL = 7e-4f;

struct FactorDev {
    const float *A;
    float *Xout;
    float *X32b;        // second fp32 X buffer (workspace); X is kept in fp32 in every precision tier
    float *M32[2];
    float *T32;
    float *T432;
    double *M64[2];
    double *T64;
    double *T464;
    float *pv[3];       // Lanczos vectors: the current one, the one before it, and A times the current one
    float2 *pm_partial; // per mat-vec workgroup: (sum y^2, sum y v)
    float2 *pm_partial2; // per mat-vec workgroup, first step only: (sum a_ij^2, sum a_ii)
    float *partial;     // per lower-triangle tile: sum (M - I)^2 (2 ntri entries: a second one per tile for kernels that split tiles)
    int n, lda, ldx;
    int ld32, ld64;
    int ntri;           // lower-triangle tiles
    int tile_start;     // first tile of this factor in tile-indexed launches
    int pm_blocks;
    int pm_block_start;
    float eps_in;
    int a_packed;       // A lies in packed lower tiles (gemm.h, packed_off): lda unused
    float *pm_tile;     // packed A: per lower tile 2 x 128 partial products of the mat-vec and (sum a^2, trace part)
};
constexpr int PM_TILE_WORDS = 2 * PACK_T + 2;   // floats per tile in pm_tile

struct FactorScal {
    float lam;       // lambda_max estimate
    float eps;       // absolute eps used
    float scale;     // s
    float resid;     // last ||M - I||_F
    float inv_norm;  // 1 / ||v|| of the current Lanczos vector (the vectors are stored unnormalised)
    float inv_prev;  // the same for the vector before it
    float rho;       // largest Ritz value so far: the lambda_max estimate
    int lz_small;    // consecutive steps that moved the estimate by less than the tolerance
    int iters;       // X updates performed / scheduled
    int xloc;        // 0: current fp32 X in Xout, 1: in X32b
    int info;
    int pm_done;
    float lo, hi;    // interval assumed to contain the spectrum of the current M
    float ca, cg;    // coefficients of the current T = ca I - cg M
    float coef_next[2];   // coefficients the M-update epilogue uses for the next T
    float fro2, trace;    // ||A||_F^2 and tr(A), gathered during the first mat-vec of the lambda_max estimate
    float x_scale;        // power of two that brings X into the fp16 range for the 16-bit products
    // (lo, hi) of the M the current iteration starts from and the g of its T: lo, hi, ca, cg above
    // are advanced to the next iteration's before the products of the current one run
    float lo_cur, hi_cur, cg_cur;
    float lz_a[LZ_MAX], lz_b[LZ_MAX];   // the Lanczos recurrence: diagonal and off-diagonal of the tridiagonal matrix
};

// Scale of M, T, T^2, T^4 in the fp16-split products: their entries stay below a^4 < 23 (a <= 2.2),
// so 2^10 keeps them under 2^15 with the fp16 range ending at 65504.
constexpr float ROOT_F16_SCALE = 1024.0f;

__device__ __forceinline__ float hash_unit(uint32_t f, uint32_t j)
{
    uint32_t x = j * 0x9E3779B1u + f * 0x85EBCA77u + 0x165667B1u;
    x ^= x >> 15; x *= 0x2C1B3C6Du; x ^= x >> 12; x *= 0x297A2D39u; x ^= x >> 15;
    return (float)(x >> 8) * (1.0f / 8388608.0f) - 1.0f;   // [-1, 1)
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ---- lambda_max: Lanczos process --------------------------------------------------------------
// v_0 a fixed pseudo-random vector; step j: y = A v_j (the mat-vec kernels below), alpha_j = v_j^T y,
// w = y - alpha_j v_j - beta_{j-1} v_{j-1}, beta_j = ||w||, v_{j+1} = w / beta_j.  The estimate is the
// largest eigenvalue of the tridiagonal matrix (alpha, beta) of the steps so far: it rises monotonically
// to lambda_max and gets there in about 1 / sqrt(gap) steps where plain power iteration needs 1 / gap (a
// statistic whose leading eigenvalues lie 1 % apart: 30 - 40 steps for 1e-5, against 2e-3 after 256 power
// steps).  No re-orthogonalisation: what fp32 round-off does to the later vectors produces copies of
// converged Ritz values, never one above lambda_max by more than round-off.
// one workgroup (256 threads) per factor: start vector and its norm
__global__ __launch_bounds__(256) void pm_init_kernel(const FactorDev *fd, FactorScal *fs)
{
    const int f = blockIdx.x;
    const FactorDev &F = fd[f];
    __shared__ float red[4];
    float s = 0.0f;
    for (int j = threadIdx.x; j < F.n; j += 256) {
        // the same start vector for every factor: a factor's result does not depend on its place in the batch
        const float v = hash_unit(0u, (uint32_t)j);
        F.pv[0][j] = v;
        s += v * v;
    }
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float t = red[0] + red[1] + red[2] + red[3];
        fs[f].inv_norm = t > 0.0f ? rsqrtf(t) : 0.0f;
        fs[f].inv_prev = 0.0f;
        fs[f].rho = 0.0f;
        fs[f].lz_small = 0;
        fs[f].pm_done = 0;
    }
}

// y = A v for PM_ROWS rows of one factor; v = v_raw * inv_norm on the fly.
// Grid: x = row block, y = factor - a finished factor's workgroups leave after two loads, which
// keeps the launches that follow a factor's convergence cheap.
__global__ __launch_bounds__(256) void pm_matvec_kernel(const FactorDev *fd, const FactorScal *fs,
                                                        int nf, int src, int dst, int first)
{
    const int lo = blockIdx.y;
    if (fs[lo].pm_done) return;
    const FactorDev &F = fd[lo];
    if (F.a_packed) return;                  // packed statistics take the tile kernels below
    const int blk = (int)blockIdx.x;
    if (blk >= F.pm_blocks) return;
    const int n = F.n, lda = F.lda;
    const float *__restrict__ v = F.pv[src];
    float *__restrict__ y = F.pv[dst];
    const float inv = fs[lo].inv_norm;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool vec_ok = ((reinterpret_cast<uintptr_t>(F.A) & 15u) == 0) && ((lda & 3) == 0);
    __shared__ float red[4][4];
    float syy = 0.0f, syv = 0.0f, saa = 0.0f, str = 0.0f;
    for (int rr = 0; rr < PM_ROWS / 4; ++rr) {
        const int row = blk * PM_ROWS + wave * (PM_ROWS / 4) + rr;
        if (row >= n) break;
        const float *__restrict__ a = F.A + (size_t)row * lda;
        float s = 0.0f, q = 0.0f;   // q: sum of squares of the row (first step only uses it)
        if (vec_ok) {
            const int n4 = n >> 2;
            for (int j = lane; j < n4; j += 64) {
                const float4 av = reinterpret_cast<const float4 *>(a)[j];
                const float4 vv = reinterpret_cast<const float4 *>(v)[j];
                s += av.x * vv.x + av.y * vv.y + av.z * vv.z + av.w * vv.w;
                q += av.x * av.x + av.y * av.y + av.z * av.z + av.w * av.w;
            }
            for (int j = (n4 << 2) + lane; j < n; j += 64) { s += a[j] * v[j]; q += a[j] * a[j]; }
        } else {
            for (int j = lane; j < n; j += 64) { s += a[j] * v[j]; q += a[j] * a[j]; }
        }
        s = wave_sum(s) * inv;
        if (first) q = wave_sum(q);
        if (lane == 0) {
            y[row] = s;
            syy += s * s;
            syv += s * (v[row] * inv);
            saa += q;
            str += a[row];
        }
    }
    if (lane == 0) { red[0][wave] = syy; red[1][wave] = syv; red[2][wave] = saa; red[3][wave] = str; }
    __syncthreads();
    if (threadIdx.x == 0) {
        F.pm_partial[blk] = make_float2(red[0][0] + red[0][1] + red[0][2] + red[0][3],
                                        red[1][0] + red[1][1] + red[1][2] + red[1][3]);
        if (first)
            F.pm_partial2[blk] = make_float2(red[2][0] + red[2][1] + red[2][2] + red[2][3],
                                             red[3][0] + red[3][1] + red[3][2] + red[3][3]);
    }
}

// ---- the same mat-vec for statistics in packed lower tiles -----------------------------------
// One workgroup per stored tile (ti, tj), tj <= ti: it serves both the rows of block ti (T v_tj) and,
// off the diagonal, the rows of block tj (T^T v_ti), so every element is read once.  The partial
// products go to the factor's pm_tile array and are summed in a fixed order by pm_packed_reduce_kernel
// (no atomics: the result does not depend on the order in which workgroups finish).
__global__ __launch_bounds__(256) void pm_packed_tile_kernel(const FactorDev *fd, const FactorScal *fs, int src, int first)
{
    const int f = blockIdx.y;
    if (fs[f].pm_done) return;
    const FactorDev &F = fd[f];
    if (!F.a_packed || (int)blockIdx.x >= F.ntri) return;
    int ti, tj;
    tri_decode((int)blockIdx.x, ti, tj);
    const int n = F.n;
    const float *__restrict__ tile = F.A + (size_t)blockIdx.x * PACK_T * PACK_T;
    const float *__restrict__ v = F.pv[src];
    float *out = F.pm_tile + (size_t)blockIdx.x * PM_TILE_WORDS;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c0 = tj * PACK_T + 2 * lane, r0 = ti * PACK_T;
    __shared__ float colp[4][PACK_T];
    __shared__ float red[2][4];
    // this lane's two columns of the tile: entries of v_tj, zero beyond n
    const float vj0 = c0 < n ? v[c0] : 0.0f, vj1 = c0 + 1 < n ? v[c0 + 1] : 0.0f;
    float cs0 = 0.0f, cs1 = 0.0f, saa = 0.0f, str = 0.0f;
    for (int rr = 0; rr < PACK_T / 4; ++rr) {
        const int r = wave * (PACK_T / 4) + rr, gr = r0 + r;
        float2 a = *reinterpret_cast<const float2 *>(tile + (size_t)r * PACK_T + 2 * lane);
        if (gr >= n) { a.x = 0.0f; a.y = 0.0f; }               // padding of a ragged last tile row is undefined
        if (c0 >= n) a.x = 0.0f;
        if (c0 + 1 >= n) a.y = 0.0f;
        float s = wave_sum(a.x * vj0 + a.y * vj1);
        if (lane == 0) out[r] = s;                              // row part: (T v_tj)[r]
        const float vi = gr < n ? v[gr] : 0.0f;
        cs0 += a.x * vi; cs1 += a.y * vi;                       // column part: (T^T v_ti)[c]
        if (first) {
            saa += a.x * a.x + a.y * a.y;
            if (ti == tj) { if (gr == c0) str += a.x; if (gr == c0 + 1) str += a.y; }
        }
    }
    colp[wave][2 * lane] = cs0; colp[wave][2 * lane + 1] = cs1;
    if (first) {
        saa = wave_sum(saa); str = wave_sum(str);
        if (lane == 0) { red[0][wave] = saa; red[1][wave] = str; }
    }
    __syncthreads();
    if (threadIdx.x < PACK_T)
        out[PACK_T + threadIdx.x] = colp[0][threadIdx.x] + colp[1][threadIdx.x] + colp[2][threadIdx.x] + colp[3][threadIdx.x];
    if (first && threadIdx.x == 0) {
        // an off-diagonal tile stands for its mirror image too
        const float w = ti == tj ? 1.0f : 2.0f;
        out[2 * PACK_T] = w * (red[0][0] + red[0][1] + red[0][2] + red[0][3]);
        out[2 * PACK_T + 1] = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    }
}

// y[rows of block I] = sum over tj <= I of the row parts of tile (I, tj) + sum over ti > I of the column
// parts of tile (ti, I), scaled by 1 / ||v||; per block the same partial sums pm_matvec_kernel leaves.
__global__ __launch_bounds__(PACK_T) void pm_packed_reduce_kernel(const FactorDev *fd, const FactorScal *fs, int src, int dst, int first)
{
    const int f = blockIdx.y;
    if (fs[f].pm_done) return;
    const FactorDev &F = fd[f];
    const int T = (F.n + PACK_T - 1) / PACK_T, I = (int)blockIdx.x;
    if (!F.a_packed || I >= T) return;
    const int i = threadIdx.x, row = I * PACK_T + i;
    const float inv = fs[f].inv_norm;
    const float *__restrict__ v = F.pv[src];
    float s = 0.0f, saa = 0.0f, str = 0.0f;
    for (int tj = 0; tj <= I; ++tj) {
        const float *p = F.pm_tile + (size_t)(I * (I + 1) / 2 + tj) * PM_TILE_WORDS;
        s += p[i];
        if (first && i == 0) { saa += p[2 * PACK_T]; str += p[2 * PACK_T + 1]; }
    }
    for (int ti = I + 1; ti < T; ++ti) s += F.pm_tile[(size_t)(ti * (ti + 1) / 2 + I) * PM_TILE_WORDS + PACK_T + i];
    s *= inv;
    float syy = 0.0f, syv = 0.0f;
    if (row < F.n) {
        F.pv[dst][row] = s;
        syy = s * s;
        syv = s * (v[row] * inv);
    }
    __shared__ float red[2][PACK_T / 64];
    syy = wave_sum(syy); syv = wave_sum(syv);
    if ((i & 63) == 0) { red[0][i >> 6] = syy; red[1][i >> 6] = syv; }
    __syncthreads();
    if (i == 0) {
        F.pm_partial[I] = make_float2(red[0][0] + red[0][1], red[1][0] + red[1][1]);
        // the off-diagonal tiles of the block rows below this one were counted there (weight 2)
        if (first) F.pm_partial2[I] = make_float2(saa, str);
    }
}

// Largest eigenvalue of the symmetric tridiagonal matrix with diagonal a[0 .. m) and off-diagonal
// b[0 .. m - 1), by bisection on the number of eigenvalues below x (signs of the pivots of T - x I).
__device__ double tridiag_largest(const float *a, const float *b, int m)
{
    double lo = (double)a[0], hi = lo;
    for (int i = 0; i < m; ++i) {
        const double r = (i > 0 ? fabs((double)b[i - 1]) : 0.0) + (i + 1 < m ? fabs((double)b[i]) : 0.0);
        lo = fmax(lo, (double)a[i]);               // the largest eigenvalue is at least every diagonal entry
        hi = fmax(hi, (double)a[i] + r);           // ... and at most the largest Gershgorin bound
    }
    if (m == 1 || !(hi > lo)) return lo;
    for (int it = 0; it < 48; ++it) {
        const double x = 0.5 * (lo + hi);
        int below = 0;
        double d = 1.0;
        for (int i = 0; i < m; ++i) {
            const double bb = i > 0 ? (double)b[i - 1] * (double)b[i - 1] : 0.0;
            d = (double)a[i] - x - (i > 0 ? bb / d : 0.0);
            if (d == 0.0) d = -1e-300;
            if (d < 0.0) ++below;
        }
        if (below == m) hi = x; else lo = x;
    }
    return 0.5 * (lo + hi);
}

// One workgroup per factor, after the mat-vec of step `it` (y = A v in pv[dst], v in pv[src], the vector
// before it in pv[prev]): alpha, the next Lanczos vector (over y, unnormalised), beta, the estimate, the stop.
// A factor stops once two consecutive steps have raised the estimate by less than tol2 of it (or the
// recurrence ends: beta = 0, an invariant subspace, where the estimate is exact).
__global__ __launch_bounds__(256) void pm_lanczos_kernel(const FactorDev *fd, FactorScal *fs, float tol2, int it,
                                                         int src, int dst, int prev, int first, int last)
{
    const int f = blockIdx.x;
    FactorScal &S = fs[f];
    if (S.pm_done) return;
    const FactorDev &F = fd[f];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float inv = S.inv_norm, inv_p = S.inv_prev;
    const float beta_p = it > 0 ? S.lz_b[it - 1] : 0.0f;
    __shared__ double red[4][4];
    // sums the mat-vec workgroups left per block of rows, in a fixed order
    double yy = 0.0, yv = 0.0, aa = 0.0, tr = 0.0;
    for (int b = tid; b < F.pm_blocks; b += 256) {
        const float2 p = F.pm_partial[b];
        yy += (double)p.x; yv += (double)p.y;
        if (first) { const float2 q = F.pm_partial2[b]; aa += (double)q.x; tr += (double)q.y; }
    }
    auto block_sum4 = [&](double &x0, double &x1, double &x2, double &x3) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            x0 += __shfl_xor(x0, off, 64); x1 += __shfl_xor(x1, off, 64);
            x2 += __shfl_xor(x2, off, 64); x3 += __shfl_xor(x3, off, 64);
        }
        __syncthreads();
        if (lane == 0) { red[0][wave] = x0; red[1][wave] = x1; red[2][wave] = x2; red[3][wave] = x3; }
        __syncthreads();
        x0 = red[0][0] + red[0][1] + red[0][2] + red[0][3]; x1 = red[1][0] + red[1][1] + red[1][2] + red[1][3];
        x2 = red[2][0] + red[2][1] + red[2][2] + red[2][3]; x3 = red[3][0] + red[3][1] + red[3][2] + red[3][3];
    };
    block_sum4(yy, yv, aa, tr);
    const bool finite = (yy == yy) && (yy < 3.0e38);
    const float alpha = (float)yv;                    // v is a unit vector: alpha = v^T A v
    // w = y - alpha v - beta_{j-1} v_{j-1}, written over y
    const float *__restrict__ v = F.pv[src], *__restrict__ vp = F.pv[prev];
    float *__restrict__ w = F.pv[dst];
    double ww = 0.0, z1 = 0.0, z2 = 0.0, z3 = 0.0;
    if (finite) {
        for (int i = tid; i < F.n; i += 256) {
            float x = w[i] - alpha * (v[i] * inv);
            if (it > 0) x -= beta_p * (vp[i] * inv_p);
            w[i] = x;
            ww += (double)x * (double)x;
        }
    }
    block_sum4(ww, z1, z2, z3);
    if (tid != 0) return;
    if (first) { S.fro2 = (float)aa; S.trace = (float)tr; }
    if (!finite) { S.rho = NAN; S.pm_done = 1; return; }
    const float beta = (float)sqrt(ww);
    S.lz_a[it] = alpha;
    S.lz_b[it] = beta;
    const double theta = tridiag_largest(S.lz_a, S.lz_b, it + 1);
    const double before = (double)S.rho;
    S.rho = (float)theta;
    // breakdown: A v stayed in the span of the vectors so far (a multiple of the identity, a start vector
    // that is an eigenvector, rank deficiency exhausted): the largest Ritz value is an eigenvalue
    const bool ended = !(beta > 1e-7f * fabsf((float)theta)) || !(beta > 0.0f);
    if (it > 0 && theta - before <= (double)tol2 * fabs(theta)) S.lz_small += 1; else S.lz_small = 0;
    if (ended || S.lz_small >= 2 || last) { S.pm_done = 1; return; }
    S.inv_prev = inv;
    S.inv_norm = 1.0f / beta;
}

// ---- scaling and start of the coupled iteration ---------------------------------------------
__global__ void root_setup_kernel(const FactorDev *fd, FactorScal *fs, int *state, int nf,
                                  int relative, float margin, int root, int adapted)
{
    const int f = blockIdx.x * blockDim.x + threadIdx.x;
    if (f >= nf) return;
    FactorScal &S = fs[f];
    const float lam = S.rho;
    S.lam = lam;
    S.iters = 0;
    S.xloc = 0;
    S.resid = 0.0f;
    const float eps = relative ? fd[f].eps_in * lam : fd[f].eps_in;
    S.eps = eps;
    const float denom = (1.0f + margin) * lam + eps;
    const bool ok = (lam == lam) && (lam >= 0.0f) && (lam < 3.0e38f) && (denom > 0.0f) && (denom < 3.0e38f);
    if (!ok) {
        S.scale = 0.0f;
        S.info = ASTERIA_INFO_NOT_PD;
        state[f] = ST_FAIL;
    } else {
        S.scale = 1.0f / denom;
        S.info = ASTERIA_INFO_OK;
        state[f] = ST_RUN;
    }
    // spectrum of M_0 = s (A + eps I): at most 1 by the scaling; at least eps s for a positive
    // semi-definite A (halved: round-off in the statistics may push eigenvalues slightly below 0)
    double lo = ok ? 0.5 * (double)eps / (double)denom : 1.0;
    if (!(lo > 1e-12)) lo = 1e-12;
    if (ok) {
        // ||M_0 - I||_F^2 = s^2 ||A + eps I||_F^2 - 2 s tr(A + eps I) + n bounds every |mu - 1|:
        // a well-conditioned factor gets a much tighter interval than [eps s, 1]
        const double sc = 1.0 / (double)denom, e = (double)eps, n = (double)fd[f].n;
        const double f2 = (double)S.fro2 + 2.0 * e * (double)S.trace + n * e * e;
        const double tr = (double)S.trace + n * e;
        double r2 = sc * sc * f2 - 2.0 * sc * tr + n;
        r2 = r2 * (1.0 + 1e-3) + 1e-6 * n;           // slack for the fp32 sums
        if (r2 > 0.0 && r2 < 1.0) { const double l1 = 1.0 - sqrt(r2); if (l1 > lo) lo = l1; }
    }
    // Every iterate X_k = xs prod T_j has eigenvalues x with (x / xs)^root lambda = mu <= 2, lambda >= lo
    // an eigenvalue of M_0 and mu the matching one of M_k: |X_k| <= xs (2 / lo)^(1/root).  The
    // fp16-split products scale X by the largest power of two that keeps this bound below 30000.
    {
        const double xs = ok ? pow((double)S.scale, 1.0 / (double)root) : 1.0;
        const double bound = xs * pow(2.0 / lo, 1.0 / (double)root);
        int e = (int)floor(log2(30000.0 / bound));
        e = e < -60 ? -60 : (e > 60 ? 60 : e);
        S.x_scale = (float)ldexp(1.0, e);
    }
    double a, g;
    root_coefficients(lo, 1.0, root, adapted != 0, ROOT_THETA, a, g);
    S.lo = (float)lo; S.hi = 1.0f;
    S.ca = (float)a; S.cg = (float)g;
    S.coef_next[0] = (float)a; S.coef_next[1] = (float)g;
}

// 4 consecutive elements as 16-byte stores (the destination is 16-byte aligned)
__device__ __forceinline__ void store4(float *p, const float (&v)[4])
{
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void store4(double *p, const double (&v)[4])
{
    reinterpret_cast<double2 *>(p)[0] = make_double2(v[0], v[1]);
    reinterpret_cast<double2 *>(p)[1] = make_double2(v[2], v[3]);
}

// One workgroup per lower-triangle 128 x 128 tile: M_0, T_0, X_0 and the residual partial sums.
template <typename TC>
__global__ __launch_bounds__(256) void root_init_kernel(const FactorDev *fd, const FactorScal *fs,
                                                        const int *state, int nf, int total_tiles,
                                                        int root)
{
    const int t_global = blockIdx.x;
    if (t_global >= total_tiles) return;
    int lo = 0, hi = nf - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (fd[mid].tile_start <= t_global) lo = mid; else hi = mid - 1;
    }
    const FactorDev &F = fd[lo];
    if (state[lo] != ST_RUN) return;
    const int lt = t_global - F.tile_start;
    int ti, tj;
    tri_decode(lt, ti, tj);
    const int n = F.n, lda = F.lda;
    const TC s = (TC)fs[lo].scale;
    const TC eps = (TC)fs[lo].eps;
    const TC xs = (TC)pow((double)fs[lo].scale, 1.0 / (double)root);
    const TC ca = (TC)fs[lo].ca, cg = (TC)fs[lo].cg;
    // X_0 = xs I is never stored: the first update X_1 = X_0 T_0 = xs T_0 is written directly
    // (into the buffer that holds X after an odd number of updates), which saves one product.
    TC *M, *T;
    int ldm;
    if (sizeof(TC) == 8) {
        M = reinterpret_cast<TC *>(F.M64[0]); T = reinterpret_cast<TC *>(F.T64); ldm = F.ld64;
    } else {
        M = reinterpret_cast<TC *>(F.M32[0]); T = reinterpret_cast<TC *>(F.T32); ldm = F.ld32;
    }
    float *X = F.X32b;            // holds X after an odd number of updates
    // no fp32 copy of T_0 is needed: X_1 = xs T_0 is written here, and the first X product (k = 1)
    // reads the fp32 T_1 that the M-update epilogue of iteration 0 writes
    const int ldx = F.ld32;
    // The tile pair (ti, tj) / (tj, ti) is walked in 32 x 32 sub-tiles.  P = A[sub(ti, tj)] and
    // Q = A[sub(tj, ti)] are both read along rows (coalesced) into LDS; the symmetrised value at
    // (r, c) of tile (ti, tj) is (P[r][c] + Q[c][r]) / 2 and the one at (c, r) of tile (tj, ti) is
    // the same number, so every global read and write of this kernel runs along rows.
    float rsum = 0.0f;
    __shared__ float red[4];
    // Full tiles with 16-byte aligned rows: 64 x 64 sub-tiles, 16-byte global loads, and 32-byte
    // (fp64) or 16-byte (fp32) stores of 4 consecutive elements per thread; LDS rows of 65 words
    // keep both the row-wise and the transposed reads free of bank conflicts.
    // Packed lower tiles: tile (ti, tj) is stored once, dense with 128 floats per row, and stands for
    // its mirror image; the value at (r, c) is the stored one (nothing to symmetrise).
    const bool packed = F.a_packed != 0;
    const float *Ap = packed ? F.A + (size_t)lt * PACK_T * PACK_T : nullptr;
    const bool aligned = ti * BM + BM <= n && (packed || ((lda & 3) == 0 && (reinterpret_cast<uintptr_t>(F.A) & 15u) == 0));
    if (aligned) {
        __shared__ float Pw[64][65], Qw[64][65];
        const int g = threadIdx.x & 15, rw = threadIdx.x >> 4;     // 16 column groups of 4 x 16 rows
        for (int sub = 0; sub < 4; ++sub) {
            const int si = sub >> 1, sj = sub & 1;
            if (ti == tj && si < sj) continue;                       // covered by the mirrored sub-tile
            const int r0 = ti * BM + si * 64, c0 = tj * BN + sj * 64;
            const bool diag_sub = (ti == tj && si == sj);
            __syncthreads();
            for (int rr = rw; rr < 64; rr += 16) {
                const float4 pv = packed ? *reinterpret_cast<const float4 *>(Ap + (size_t)(si * 64 + rr) * PACK_T + sj * 64 + 4 * g)
                                         : *reinterpret_cast<const float4 *>(F.A + (size_t)(r0 + rr) * lda + c0 + 4 * g);
                Pw[rr][4 * g] = pv.x; Pw[rr][4 * g + 1] = pv.y; Pw[rr][4 * g + 2] = pv.z; Pw[rr][4 * g + 3] = pv.w;
                if (!packed) {
                    const float4 qv = *reinterpret_cast<const float4 *>(F.A + (size_t)(c0 + rr) * lda + r0 + 4 * g);
                    Qw[rr][4 * g] = qv.x; Qw[rr][4 * g + 1] = qv.y; Qw[rr][4 * g + 2] = qv.z; Qw[rr][4 * g + 3] = qv.w;
                }
            }
            __syncthreads();
            for (int rr = rw; rr < 64; rr += 16) {
                // elements (r, c .. c + 3) of tile (ti, tj)
                {
                    const int r = r0 + rr, c = c0 + 4 * g;
                    TC mv[4], tv[4];
                    float xv[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const TC av = packed ? (TC)Pw[rr][4 * g + e] : (TC)0.5 * ((TC)Pw[rr][4 * g + e] + (TC)Qw[4 * g + e][rr]);
                        const TC d = (r == c + e) ? (TC)1 : (TC)0;
                        mv[e] = s * (av + eps * d);
                        tv[e] = ca * d - cg * mv[e];
                        xv[e] = (float)(xs * tv[e]);
                        const float er = (float)(mv[e] - d);
                        rsum += diag_sub ? er * er : 2.0f * er * er;
                    }
                    store4(M + (size_t)r * ldm + c, mv);
                    store4(T + (size_t)r * ldm + c, tv);
                    store4(X + (size_t)r * ldx + c, xv);
                }
                // elements (r2, c2 .. c2 + 3) of the mirrored tile (tj, ti): the same numbers transposed
                if (!diag_sub) {
                    const int r2 = c0 + rr, c2 = r0 + 4 * g;
                    TC mv[4], tv[4];
                    float xv[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const TC av = packed ? (TC)Pw[4 * g + e][rr] : (TC)0.5 * ((TC)Pw[4 * g + e][rr] + (TC)Qw[rr][4 * g + e]);
                        mv[e] = s * av;                              // off the diagonal: no eps, d = 0
                        tv[e] = -cg * mv[e];
                        xv[e] = (float)(xs * tv[e]);
                    }
                    store4(M + (size_t)r2 * ldm + c2, mv);
                    store4(T + (size_t)r2 * ldm + c2, tv);
                    store4(X + (size_t)r2 * ldx + c2, xv);
                }
            }
        }
        rsum = wave_sum(rsum);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = rsum;
        __syncthreads();
        if (threadIdx.x == 0) { F.partial[lt] = red[0] + red[1] + red[2] + red[3]; F.partial[F.ntri + lt] = 0.0f; }
        return;
    }
    __shared__ float Ps[32][33], Qs[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8 threads
    for (int sub = 0; sub < 16; ++sub) {
        const int si = sub >> 2, sj = sub & 3;
        const int r0 = ti * BM + si * 32, c0 = tj * BN + sj * 32;
        if (r0 >= n || c0 >= n) continue;                        // uniform over the workgroup
        if (ti == tj && si < sj) continue;                       // covered by the mirrored sub-tile
        __syncthreads();
        for (int rr = ty; rr < 32; rr += 8) {
            const int r = r0 + rr, c = c0 + tx;
            Ps[rr][tx] = (r < n && c < n) ? (packed ? Ap[(size_t)(si * 32 + rr) * PACK_T + sj * 32 + tx] : F.A[(size_t)r * lda + c]) : 0.0f;
            const int r2 = c0 + rr, c2 = r0 + tx;                // sub-tile (sj, si) of tile (tj, ti)
            if (!packed) Qs[rr][tx] = (r2 < n && c2 < n) ? F.A[(size_t)r2 * lda + c2] : 0.0f;
        }
        __syncthreads();
        const bool diag_sub = (ti == tj && si == sj);
        for (int rr = ty; rr < 32; rr += 8) {
            // element (r, c) of tile (ti, tj)
            {
                const int r = r0 + rr, c = c0 + tx;
                if (r < n && c < n) {
                    const TC av = packed ? (TC)Ps[rr][tx] : (TC)0.5 * ((TC)Ps[rr][tx] + (TC)Qs[tx][rr]);
                    const TC d = (r == c) ? (TC)1 : (TC)0;
                    const TC m = s * (av + eps * d);
                    const TC t = ca * d - cg * m;
                    M[(size_t)r * ldm + c] = m;
                    T[(size_t)r * ldm + c] = t;
                    X[(size_t)r * ldx + c] = (float)(xs * t);
                    const float e = (float)(m - d);
                    // a diagonal sub-tile holds both triangles itself; every other one stands for two
                    rsum += diag_sub ? e * e : 2.0f * e * e;
                }
            }
            // element (r2, c2) of the mirrored tile (tj, ti): same value, written along its own rows
            if (!diag_sub) {
                const int r2 = c0 + rr, c2 = r0 + tx;
                if (r2 < n && c2 < n) {
                    const TC av = packed ? (TC)Ps[tx][rr] : (TC)0.5 * ((TC)Ps[tx][rr] + (TC)Qs[rr][tx]);
                    const TC m = s * av;                          // off the diagonal: no eps, d = 0
                    const TC t = -cg * m;
                    M[(size_t)r2 * ldm + c2] = m;
                    T[(size_t)r2 * ldm + c2] = t;
                    X[(size_t)r2 * ldx + c2] = (float)(xs * t);
                }
            }
        }
    }
    rsum = wave_sum(rsum);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = rsum;
    __syncthreads();
    if (threadIdx.x == 0) { F.partial[lt] = red[0] + red[1] + red[2] + red[3]; F.partial[F.ntri + lt] = 0.0f; }
}

// One wavefront per factor, run before iteration k (and once after the last one with
// final_pass = 1): evaluates the residual of running factors and advances the state machine.
__global__ __launch_bounds__(64) void root_control_kernel(const FactorDev *fd, FactorScal *fs, int *state,
                                                          int k, int fp32_phase, int final_pass,
                                                          float stop_resid, int root, int adapted, int look_ahead)
{
    const int f = blockIdx.x;
    const FactorDev &F = fd[f];
    FactorScal &S = fs[f];
    int st = state[f];
    if (st == ST_DONE || st == ST_FAIL) return;
    if (st == ST_LAST) {
        st = ST_DONE;
    } else {
        float r2 = 0.0f;
        // the int8 product writes two partial sums per tile (one per half), the other kernels the
        // first only: the second is cleared once read
        for (int i = threadIdx.x; i < F.ntri; i += 64) {
            r2 += F.partial[i] + F.partial[F.ntri + i];
            F.partial[F.ntri + i] = 0.0f;
        }
        r2 = wave_sum(r2);
        const float resid = sqrtf(r2);
        if (!(r2 == r2) || !(r2 < 3.0e38f)) {
            st = ST_FAIL;
            if (threadIdx.x == 0) { S.info = ASTERIA_INFO_NOT_PD; S.resid = resid; }
        } else {
            if (threadIdx.x == 0) S.resid = resid;
            // Last X update now?  X_{k+1} = X_k T_k differs from the root by |mu - 1| / 4 per eigen-
            // direction, mu in the spectrum of M_{k+1}.  Three ways to know that this is small:
            //  - the measured residual of M_k is below stop_resid (the update squares it);
            //  - the interval predicted for M_k has contracted to 1 +- ROOT_STOP_DEV;
            //  - the image of that interval under this iteration's map, i.e. the interval of
            //    M_{k+1}, lies within 1 +- 4 ROOT_X_TOL: M_{k+1} need not be formed at all.
            // The predictions are trusted only while the measured residual is consistent with
            // them: every |mu - 1| is at most ||M_k - I||_F, so an eigenvalue far outside shows.
            const float dev = fmaxf(1.0f - S.lo, S.hi - 1.0f);
            const bool consistent = resid < 1.5f * sqrtf((float)F.n) * dev + 2e-3f;
            double lo_k = (double)S.lo, hi_k = (double)S.hi;
            const double rb = (double)resid * 1.001 + 1e-5;
            if (1.0 - rb > lo_k) lo_k = 1.0 - rb;
            if (1.0 + rb < hi_k) hi_k = 1.0 + rb;
            if (!(hi_k > lo_k)) { lo_k = 1.0 - rb; hi_k = 1.0 + rb; }
            const RootInterval nx = root_image(lo_k, hi_k, root, (double)S.ca, (double)S.cg);
            const double dev_next = fmax(1.0 - nx.lo, nx.hi - 1.0);
            const bool pred_ok = consistent && dev < ROOT_STOP_DEV;
            const bool ahead_ok = look_ahead && consistent && dev_next <= 4.0 * (double)ROOT_X_TOL;
            if (resid < stop_resid || pred_ok || ahead_ok) st = ST_LAST;
        }
    }
    if (threadIdx.x == 0) {
        if (!final_pass && (st == ST_RUN || st == ST_LAST)) {
            S.iters += 1;
            S.xloc = (k + 1) & 1;      // X after k + 1 updates: 1 = workspace buffer, 0 = the caller's X
        }
        if (final_pass && (st == ST_RUN || st == ST_LAST)) S.info = ASTERIA_INFO_NOT_CONVERGED;
        if (!final_pass && st == ST_RUN) {
            // iteration k will produce M_{k+1} = f(M_k) and T_{k+1}: advance the spectrum interval
            // through the scalar map and pick the coefficients of T_{k+1} for that new interval
            // every |mu - 1| is at most the measured ||M_k - I||_F: tighten the predicted interval
            double lo_k = (double)S.lo, hi_k = (double)S.hi;
            const double rb = (double)S.resid * 1.001 + 1e-5;
            if (1.0 - rb > lo_k) lo_k = 1.0 - rb;
            if (1.0 + rb < hi_k) hi_k = 1.0 + rb;
            if (!(hi_k > lo_k)) { lo_k = 1.0 - rb; hi_k = 1.0 + rb; }
            const RootInterval im = root_image(lo_k, hi_k, root, (double)S.ca, (double)S.cg);
            double a, g;
            root_coefficients(im.lo, im.hi, root, adapted != 0, ROOT_THETA, a, g);
            S.lo_cur = S.lo; S.hi_cur = S.hi; S.cg_cur = S.cg;
            S.lo = (float)im.lo; S.hi = (float)im.hi;
            S.ca = (float)a; S.cg = (float)g;
            S.coef_next[0] = (float)a; S.coef_next[1] = (float)g;
        }
        state[f] = st;
    }
}

// Copy X from the workspace buffer to the caller's X where the last fp32 update landed there,
// and publish the per-factor outcome.  One workgroup per 128 x 128 tile.
__global__ __launch_bounds__(256) void root_finalize_kernel(const FactorDev *fd, const FactorScal *fs,
                                                            const int *state, int nf, const int *sq_tile_start,
                                                            int first, int32_t *info, int32_t *iters,
                                                            float *resid, float *lambda_max)
{
    int lo = 0, hi = nf - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (sq_tile_start[mid] <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
    }
    const FactorDev &F = fd[lo];
    const FactorScal &S = fs[lo];
    const int lt = (int)blockIdx.x - sq_tile_start[lo];
    if (lt == 0 && threadIdx.x == 0) {
        if (info) info[first + lo] = S.info;
        if (iters) iters[first + lo] = S.iters;
        if (resid) resid[first + lo] = S.resid;
        if (lambda_max) lambda_max[first + lo] = S.lam;
    }
    if (state[lo] == ST_FAIL || S.xloc == 0) return;
    const int n = F.n;
    const int tpr = (n + BN - 1) / BN;
    const int ti = lt / tpr, tj = lt % tpr;
    for (int e = threadIdx.x; e < BM * BN; e += 256) {
        const int row = ti * BM + e / BN, col = tj * BN + e % BN;
        if (row >= n || col >= n) continue;
        F.Xout[(size_t)row * F.ldx + col] = F.X32b[(size_t)row * F.ld32 + col];
    }
}

// ---- host side -------------------------------------------------------------------------------
inline int ld4(int n) { return (n + 3) & ~3; }
inline int ld2(int n) { return (n + 1) & ~1; }

struct Plan {
    int max_iters;
    int fp64_iters;
    int power_iters;
    int root;
    int lowp_from;     // first iteration that may run on the fp16 matrix cores (operands split in two fp16 terms)
    float stop_resid, power_tol, margin;
    bool use64, use32, adapted, lowp_auto;
    int i8_slices;     // 0, or the number of int8 slices the products of the fp64 iterations are computed with
    bool xt_lowp;      // fully automatic precision: X updates on the fp16 cores (split operands) from the
                       // first product on, and the look-ahead stop rule (accuracy class 1e-3)
};

// Host mirror of the device-side schedule for a spectrum of M_0 in [lo0, 1]:
//   *iters  worst-case number of X updates: iterations until sqrt(n) * max|1 - mu| < stop over the
//           interval, plus the last update that follows;
//   *lead64 number of leading iterations that start while the bottom of the spectrum is still
//           below `thr` (those run in fp64 under the automatic precision rule).
// bottom of M's spectrum from which the 16-bit-split tier may run under the automatic rule
constexpr double ROOT_LOWP_FLOOR = 0.5 * 5.96e-8 / 1e-3;

void simulate_schedule(double lo0, int n, int root, bool adapted, double stop, double thr, int cap,
                       int *iters, int *lead64, double thr_lowp = 0.0, int *lead_full = nullptr)
{
    double lo = lo0, hi = 1.0;
    int k = 0, lead = 0, leadf = 0;
    while (k < cap) {
        const double dev = std::max(fabs(1.0 - lo), fabs(1.0 - hi));
        if (sqrt((double)n) * dev < stop) break;
        if (lo < thr) lead = k + 1;
        if (lo < thr_lowp) leadf = k + 1;
        double a, g;
        root_coefficients(lo, hi, root, adapted, ROOT_THETA, a, g);
        const RootInterval im = root_image(lo, hi, root, a, g);
        lo = im.lo; hi = im.hi;
        ++k;
    }
    *iters = k + 1;
    *lead64 = lead;
    if (lead_full) *lead_full = leadf;
}

// The fp32 work matrices of the M-chain (M x 2, T^4) are first written when the fp64 tier hands over - M
// by the epilogue of its last M-update, which no longer stores the fp64 T that lies there - and the
// fp64 T and T^4 are dead from then on: they share one region.
size_t shared_region_bytes(int n, bool use64, bool use32)
{
    const size_t b32 = use32 ? 3 * Carver::need((size_t)n * ld4(n), sizeof(float)) : 0;
    const size_t b64 = use64 ? 2 * Carver::need((size_t)n * ld2(n), sizeof(double)) : 0;
    return b32 > b64 ? b32 : b64;
}

size_t factor_matrix_bytes(int n, bool use64, bool use32)
{
    size_t b = 2 * Carver::need((size_t)n * ld4(n), sizeof(float));            // second X buffer, T (fp32)
    b += shared_region_bytes(n, use64, use32);                                 // fp64 T, T^4 | fp32 M x 2, T^4
    if (use64) b += 2 * Carver::need((size_t)n * ld2(n), sizeof(double));      // fp64 M x 2
    return b;
}

// sliced operands of the int8 path: two buffers of planes, row exponents and diagonals
size_t factor_i8_bytes(int n, int ns)
{
    if (ns <= 0) return 0;
    return 2 * (Carver::need(i8_plane_bytes(n, ns), 1) + Carver::need(i8_rows(n), sizeof(int)) +
                Carver::need(i8_rows(n), sizeof(double))) + Carver::need(1, sizeof(I8Factor));
}

size_t factor_small_bytes(int n)
{
    const int pmb = (n + PM_ROWS - 1) / PM_ROWS;
    return 3 * Carver::need((size_t)ld4(n), sizeof(float)) + 2 * Carver::need((size_t)pmb, sizeof(float2)) +
           Carver::need(2 * (size_t)tri_tiles(n), sizeof(float)) + Carver::need((size_t)tri_tiles(n) * PM_TILE_WORDS, sizeof(float)) +
           sizeof(FactorDev) + sizeof(FactorScal) +
           2 * sizeof(int) + 16 * sizeof(GemmProblem);
}

size_t fixed_bytes() { return 64 * 256; }   // alignment slack of the shared arrays + coefficient table

asteria_status make_plan(const asteria_root_opts *opts_in, asteria_eps_mode mode, const float *eps,
                         int eps_count, int root, Plan &pl)
{
    asteria_root_opts o;
    asteria_root_opts_default(&o);
    if (opts_in) o = *opts_in;
    if (o.max_iters <= 0 || o.power_iters <= 0) return ASTERIA_INVALID_ARG;
    if (!(o.stop_resid > 0.0f) || !(o.power_tol > 0.0f) || !(o.lambda_margin >= 0.0f)) return ASTERIA_INVALID_ARG;
    if (o.schedule != 0 && o.schedule != 1) return ASTERIA_UNSUPPORTED;
    pl.adapted = o.schedule == 1;
    pl.root = root;
    pl.max_iters = o.max_iters;
    pl.power_iters = o.power_iters;
    pl.stop_resid = o.stop_resid;
    pl.power_tol = o.power_tol;
    pl.margin = o.lambda_margin;
    int j = o.fp64_iters;
    if (j < 0) {
        // fp32 round-off of relative size u injected while the bottom of M's spectrum is mu costs
        // about u / mu in the root: stay in fp64 while 0.5 u_fp32 / mu > 1e-3, i.e. mu < 3e-5.
        if (mode == ASTERIA_EPS_RELATIVE && eps) {
            float emin = eps[0];
            for (int i = 1; i < eps_count; ++i) emin = std::min(emin, eps[i]);
            // the device starts the interval at half of eps s (round-off in the statistics may push
            // eigenvalues slightly below zero): the same start here and in the rule for lowp_from below
            const double lo0 = 0.5 * (double)emin / (1.0 + (double)pl.margin + (double)emin);
            int it = 0;
            if (emin > 0.0f) simulate_schedule(lo0, 1, root, pl.adapted, 1e-3, ROOT_LOWP_FLOOR, o.max_iters, &it, &j);
            else j = o.max_iters;
        } else {
            j = pl.adapted ? 2 : 4;   // the host cannot see eps / lambda_max here
        }
    }
    // Iterations after the fp64 prefix: products of fp32 operands split into two fp16 terms (three
    // fp16 MFMA passes) keep the operands to 2^-22, within a factor 4 of fp32, and run twice as fast
    // as the fp32 matrix cores; they take over as soon as the bottom of M's spectrum is above
    // ROOT_LOWP_FLOOR, the bound below which the automatic rule keeps fp64.
    int jl = o.lowp_from;
    if (jl < 0) {
        jl = o.max_iters;
        if (mode == ASTERIA_EPS_RELATIVE && eps) {
            float emin = eps[0];
            for (int i = 1; i < eps_count; ++i) emin = std::min(emin, eps[i]);
            if (emin > 0.0f) {
                const double lo0 = 0.5 * (double)emin / (1.0 + (double)pl.margin + (double)emin);
                int it = 0, l64 = 0;
                simulate_schedule(lo0, 1, root, pl.adapted, 1e-3, 0.0, o.max_iters, &it, &l64, ROOT_LOWP_FLOOR, &jl);
            }
        }
    }
    pl.lowp_from = jl;
    pl.lowp_auto = o.lowp_from < 0;
    // only under fully automatic precision rules, and only where they use the 16-bit tier at all
    pl.xt_lowp = pl.lowp_auto && o.fp64_iters < 0 && jl < o.max_iters;
    pl.fp64_iters = std::min(j, pl.max_iters);
    pl.use64 = pl.fp64_iters > 0;
    pl.use32 = pl.fp64_iters < pl.max_iters;
    if (o.int8_slices != -1 && o.int8_slices != 0 && o.int8_slices != 4 && o.int8_slices != 5) return ASTERIA_UNSUPPORTED;
    pl.i8_slices = pl.use64 ? (o.int8_slices < 0 ? 5 : o.int8_slices) : 0;
    return ASTERIA_OK;
}

asteria_status validate(const asteria_factor *f, int nf, int root, const float *eps, int eps_count)
{
    if (!f || nf <= 0 || !eps) return ASTERIA_INVALID_ARG;
    if (root != 2 && root != 4) return ASTERIA_UNSUPPORTED;
    if (eps_count != 1 && eps_count != nf) return ASTERIA_INVALID_ARG;
    for (int i = 0; i < eps_count; ++i)
        if (!(eps[i] >= 0.0f) || !(eps[i] < 3.0e38f)) return ASTERIA_INVALID_ARG;
    for (int i = 0; i < nf; ++i) {
        if (!f[i].A || !f[i].X || f[i].n <= 0 || f[i].ldx < f[i].n) return ASTERIA_INVALID_ARG;
        if (f[i].a_layout == ASTERIA_LAYOUT_FULL) { if (f[i].lda < f[i].n) return ASTERIA_INVALID_ARG; }
        else if (f[i].a_layout == ASTERIA_LAYOUT_PACKED) { if (reinterpret_cast<uintptr_t>(f[i].A) & 15u) return ASTERIA_INVALID_ARG; }
        else return ASTERIA_INVALID_ARG;
    }
    return ASTERIA_OK;
}

// The grouped-GEMM problem tables of one pass: [parity] X' = X T on the fp32 buffers, and
// [precision 0 = fp32, 1 = fp64][parity][T T | T^2 T^2 | T^p M] for the chain of M.
struct RootTables {
    GemmProblem *xt[2];
    GemmProblem *tab[2][2][3];
    GemmProblem *last64[2];    // [parity] the M-update of the last fp64 iteration: it hands M over in fp32
};

// one thread per factor writes its entry of every table
__global__ void root_tables_kernel(const FactorDev *__restrict__ fd, FactorScal *fs, int cnt, int root, int use32,
                                   int use64, RootTables rt, const I8Factor *xf)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= cnt) return;
    const FactorDev F = fd[i];
    const float ca = (float)(root + 1) / (float)root, cg = 1.0f / (float)root;
    GemmProblem p = {};
    p.M = p.N = p.K = F.n;
    p.state_idx = i;
    p.alpha = 1.0f; p.beta = 0.0f; p.ep_a = ca; p.ep_g = cg;
    p.flags = GEMM_SYM;
    p.tile_start = F.tile_start;
    p.sa = ROOT_F16_SCALE; p.sb = ROOT_F16_SCALE;       // read by the fp16-split kernel only
    for (int pa = 0; pa < 2; ++pa) {
        // X after an odd number of updates lives in the workspace buffer, else in the caller's X
        GemmProblem q = p;
        q.state_mask = (1 << ST_RUN) | (1 << ST_LAST);
        q.A = pa ? (const void *)F.X32b : (const void *)F.Xout; q.lda = pa ? F.ld32 : F.ldx;
        q.B = F.T32; q.ldb = F.ld32;
        q.C = pa ? (void *)F.Xout : (void *)F.X32b; q.ldc = pa ? F.ldx : F.ld32;
        q.sa_dev = &fs[i].x_scale;
        rt.xt[pa][i] = q;
    }
    p.state_mask = (1 << ST_RUN);
    for (int pr = 0; pr < 2; ++pr) {
        if ((pr == 0 && !use32) || (pr == 1 && !use64)) continue;
        for (int pa = 0; pa < 2; ++pa) {
            const void *Tm, *Mcur;
            void *Mnext, *T4, *Tw;
            int ldw;
            if (pr == 1) {
                Tm = F.T64; Tw = F.T64; Mcur = F.M64[pa]; Mnext = F.M64[pa ^ 1]; T4 = F.T464; ldw = F.ld64;
            } else {
                Tm = F.T32; Tw = F.T32; Mcur = F.M32[pa]; Mnext = F.M32[pa ^ 1]; T4 = F.T432; ldw = F.ld32;
            }
            GemmProblem q = p;
            // with the int8 path on, the fp64 launches take the products it declines
            if (pr == 1 && xf) q.gate = &xf[i].gate;
            // launch 0: T2 = T T, kept in the buffer that receives M' afterwards (root 4) or in
            // the T^4 buffer (root 2, where the M-update reads T2 while writing M')
            void *T2 = (root == 4) ? Mnext : T4;
            q.A = Tm; q.lda = ldw; q.B = Tm; q.ldb = ldw; q.C = T2; q.ldc = ldw;
            rt.tab[pr][pa][0][i] = q;
            // launch 1: T4 = T2 T2 (root 4 only)
            q.A = T2; q.B = T2; q.C = T4;
            rt.tab[pr][pa][1][i] = q;
            // launch 2: M' = T^p M, T' = a I - g M' (+ its fp32 copy in the fp64 tier), residual partial sums
            q.A = (root == 4) ? (const void *)T4 : (const void *)T2; q.B = Mcur;
            q.C = Mnext; q.C2 = Tw; q.ldc2 = ldw; q.partial = F.partial;
            if (pr == 1) { q.C3 = F.T32; q.ldc3 = F.ld32; }
            q.coef = fs[i].coef_next;
            q.flags = GEMM_SYM | GEMM_EPI_ROOT;
            rt.tab[pr][pa][2][i] = q;
            if (pr == 1 && use32) {
                // ... and when it is the last fp64 iteration: the fp64 M' and T' would never be read, the fp32
                // tier starts from M' in the buffer its parity expects (it lies over the fp64 T, which this
                // product does not read)
                q.flags |= GEMM_EPI_HANDOVER;
                q.C4 = F.M32[pa ^ 1]; q.ldc4 = F.ld32;
                rt.last64[pa][i] = q;
            }
        }
    }
}

// one pass over factors [first, first + cnt) of the size-sorted order
asteria_status run_pass(const asteria_factor *f, const std::vector<int> &order, int first, int cnt,
                        int root, asteria_eps_mode mode, const float *eps, int eps_count, const Plan &pl,
                        int32_t *info, int32_t *iters, float *resid, float *lambda_max,
                        void *ws, hipStream_t stream, bool outputs_permuted, int *perm_dev_unused)
{
    (void)outputs_permuted; (void)perm_dev_unused;
    Carver cv(ws);
    FactorDev *d_fd = cv.take<FactorDev>(cnt);
    FactorScal *d_fs = cv.take<FactorScal>(cnt);
    int *d_state = cv.take<int>(cnt);
    int *d_sq = cv.take<int>(cnt);
    GemmProblem *d_tab[2][2][3];   // [precision 0 = fp32, 1 = fp64][parity][launch T T | T^2 T^2 | T^p M]
    GemmProblem *d_xt[2];          // [parity] X' = X T on the fp32 buffers (every precision tier)
    for (int pa = 0; pa < 2; ++pa) d_xt[pa] = cv.take<GemmProblem>(cnt);
    for (int pr = 0; pr < 2; ++pr)
        for (int pa = 0; pa < 2; ++pa)
            for (int l = 0; l < 3; ++l) d_tab[pr][pa][l] = cv.take<GemmProblem>(cnt);
    GemmProblem *d_last64[2];      // [parity] M-update of the last fp64 iteration
    for (int pa = 0; pa < 2; ++pa) d_last64[pa] = cv.take<GemmProblem>(cnt);

    std::vector<FactorDev> fd(cnt);
    std::vector<int> sq(cnt);
    int tri_total = 0, sq_total = 0, pm_total = 0, pm_blocks_max = 0, tri_max = 0;
    bool any_packed = false, any_full = false;
    int n_max = 0;
    double a_min = 1.0;
    for (int i = 0; i < cnt; ++i) {
        const asteria_factor &a = f[order[first + i]];
        FactorDev &F = fd[i];
        memset(&F, 0, sizeof(F));
        const int n = a.n;
        n_max = std::max(n_max, n);
        F.A = a.A; F.Xout = a.X; F.n = n; F.lda = a.lda; F.ldx = a.ldx;
        F.ld32 = ld4(n); F.ld64 = ld2(n);
        F.ntri = tri_tiles(n);
        F.tile_start = tri_total; tri_total += F.ntri;
        const int tpr = (n + BM - 1) / BM;
        sq[i] = sq_total; sq_total += tpr * tpr;
        F.a_packed = a.a_layout == ASTERIA_LAYOUT_PACKED ? 1 : 0;
        // partial sums of the mat-vec: per block of PM_ROWS rows, or per block of 128 rows for packed tiles
        F.pm_blocks = F.a_packed ? (n + PACK_T - 1) / PACK_T : (n + PM_ROWS - 1) / PM_ROWS;
        F.pm_block_start = pm_total; pm_total += F.pm_blocks;
        if (F.a_packed) { any_packed = true; tri_max = std::max(tri_max, F.ntri); }
        else { any_full = true; pm_blocks_max = std::max(pm_blocks_max, F.pm_blocks); }
        F.eps_in = eps[eps_count == 1 ? 0 : order[first + i]];
        if (mode == ASTERIA_EPS_RELATIVE) {
            const double er = (double)F.eps_in;
            a_min = std::min(a_min, er / (1.0 + (double)pl.margin + er));
        }
        for (int v = 0; v < 3; ++v) F.pv[v] = cv.take<float>(ld4(n));
        F.pm_partial = cv.take<float2>((n + PM_ROWS - 1) / PM_ROWS);
        F.pm_partial2 = cv.take<float2>((n + PM_ROWS - 1) / PM_ROWS);
        F.pm_tile = cv.take<float>((size_t)F.ntri * PM_TILE_WORDS);
        F.partial = cv.take<float>(2 * (size_t)F.ntri);
    }
    // factors too large for exact int32 sums (never reached by the 16384 limit of the other tiers'
    // workloads) keep the fp64 cores
    const int ns8 = (pl.i8_slices > 0 && n_max <= 65536) ? pl.i8_slices : 0;
    I8Factor *d_xf = nullptr;
    std::vector<I8Factor> xfh;
    if (ns8 > 0) {
        d_xf = cv.take<I8Factor>(cnt);
        xfh.resize(cnt);
        for (int i = 0; i < cnt; ++i) {
            I8Factor &X = xfh[i];
            memset(&X, 0, sizeof(X));
            const int n = fd[i].n;
            for (int b = 0; b < 2; ++b) {
                X.planes[b] = cv.take<int8_t>(i8_plane_bytes(n, ns8));
                X.expo[b] = cv.take<int>(i8_rows(n));
                X.diag[b] = cv.take<double>(i8_rows(n));
            }
            X.n = n; X.kb = (n + 31) / 32;
        }
    }
    for (int i = 0; i < cnt; ++i) {
        FactorDev &F = fd[i];
        const size_t e32 = (size_t)F.n * F.ld32, e64 = (size_t)F.n * F.ld64;
        F.X32b = cv.take<float>(e32);
        F.T32 = cv.take<float>(e32);
        unsigned char *shared = cv.take<unsigned char>(shared_region_bytes(F.n, pl.use64, pl.use32));
        if (pl.use32) {
            const size_t step = Carver::need(e32, sizeof(float));
            F.M32[0] = reinterpret_cast<float *>(shared);
            F.M32[1] = reinterpret_cast<float *>(shared + step);
            F.T432 = reinterpret_cast<float *>(shared + 2 * step);
        }
        if (pl.use64) {
            F.T64 = reinterpret_cast<double *>(shared);
            F.T464 = reinterpret_cast<double *>(shared + Carver::need(e64, sizeof(double)));
            F.M64[0] = cv.take<double>(e64); F.M64[1] = cv.take<double>(e64);
        }
    }

    // iteration budget known on the host
    int K = pl.max_iters;
    if (mode == ASTERIA_EPS_RELATIVE && a_min > 0.0) {
        int it = 0, lead = 0;
        simulate_schedule(a_min * 0.5, n_max, root, pl.adapted, (double)pl.stop_resid, 0.0, pl.max_iters, &it, &lead);
        K = std::min(K, it + 2);
    }
    const int j64 = std::min(pl.fp64_iters, K);
    // checked up to n = 4096; beyond 16384 the automatic rule keeps the factors on the fp32 cores
    const int jlow = (pl.lowp_auto && n_max > 16384) ? K : pl.lowp_from;

    // problem tables: written on the device from the factor descriptors (the 14 tables are 11 times
    // the size of the descriptors, and host tables would travel as kernel arguments)
    ASTERIA_HIP_TRY(upload_async(d_fd, fd.data(), sizeof(FactorDev) * cnt, stream));
    ASTERIA_HIP_TRY(upload_async(d_sq, sq.data(), sizeof(int) * cnt, stream));
    RootTables rt;
    for (int pa = 0; pa < 2; ++pa) rt.xt[pa] = d_xt[pa];
    for (int pr = 0; pr < 2; ++pr)
        for (int pa = 0; pa < 2; ++pa)
            for (int l = 0; l < 3; ++l) rt.tab[pr][pa][l] = d_tab[pr][pa][l];
    for (int pa = 0; pa < 2; ++pa) rt.last64[pa] = d_last64[pa];
    if (ns8 > 0) ASTERIA_HIP_TRY(upload_async(d_xf, xfh.data(), sizeof(I8Factor) * cnt, stream));
    hipLaunchKernelGGL(root_tables_kernel, dim3((cnt + 127) / 128), dim3(128), 0, stream, d_fd, d_fs, cnt, root,
                       pl.use32 ? 1 : 0, pl.use64 ? 1 : 0, rt, d_xf);
    ASTERIA_HIP_TRY(hipGetLastError());

    // 1. lambda_max
    hipLaunchKernelGGL(pm_init_kernel, dim3(cnt), dim3(256), 0, stream, d_fd, d_fs);
    const int ctl_blocks = (cnt + 127) / 128;
    const int lz_steps = std::min(pl.power_iters, LZ_MAX);
    for (int it = 0; it < lz_steps; ++it) {
        // the three vectors rotate: v_j in src, A v_j (then v_{j+1}) in dst, v_{j-1} in prev
        const int src = it % 3, dst = (it + 1) % 3, prev = (it + 2) % 3, first = it == 0 ? 1 : 0;
        if (any_full)
            hipLaunchKernelGGL(pm_matvec_kernel, dim3(pm_blocks_max, cnt), dim3(256), 0, stream, d_fd, d_fs, cnt, src, dst, first);
        if (any_packed) {
            hipLaunchKernelGGL(pm_packed_tile_kernel, dim3(tri_max, cnt), dim3(256), 0, stream, d_fd, d_fs, src, first);
            hipLaunchKernelGGL(pm_packed_reduce_kernel, dim3((n_max + PACK_T - 1) / PACK_T, cnt), dim3(PACK_T), 0, stream, d_fd, d_fs, src, dst, first);
        }
        hipLaunchKernelGGL(pm_lanczos_kernel, dim3(cnt), dim3(256), 0, stream, d_fd, d_fs, pl.power_tol * pl.power_tol, it,
                           src, dst, prev, first, it + 1 == lz_steps ? 1 : 0);
    }
    // 2. scaling, start
    hipLaunchKernelGGL(root_setup_kernel, dim3(ctl_blocks), dim3(128), 0, stream, d_fd, d_fs, d_state, cnt,
                       mode == ASTERIA_EPS_RELATIVE ? 1 : 0, pl.margin, root, pl.adapted ? 1 : 0);
    if (j64 > 0)
        hipLaunchKernelGGL(root_init_kernel<double>, dim3(tri_total), dim3(256), 0, stream, d_fd, d_fs, d_state,
                           cnt, tri_total, root);
    else
        hipLaunchKernelGGL(root_init_kernel<float>, dim3(tri_total), dim3(256), 0, stream, d_fd, d_fs, d_state,
                           cnt, tri_total, root);
    ASTERIA_HIP_TRY(hipGetLastError());

    // 3. coupled iteration
    for (int k = 0; k < K; ++k) {
        const bool p32 = k >= j64;
        hipLaunchKernelGGL(root_control_kernel, dim3(cnt), dim3(64), 0, stream, d_fd, d_fs, d_state, k,
                           p32 ? 1 : 0, 0, pl.stop_resid, root, pl.adapted ? 1 : 0, pl.xt_lowp ? 1 : 0);
        const int pa = k & 1;
        const bool lowp = p32 && k >= jlow;
        // X' = X T (X_1 comes from the start kernel).  X only needs the accuracy of the result, so
        // the update runs on the fp16 cores with split operands (22 bits) whenever the low-precision
        // tier is chosen automatically, from the first product on; otherwise with the tier of M.
        if (k > 0) {
            if (pl.xt_lowp || lowp)
                ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2, true>(d_xt[pa], cnt, tri_total, d_state, stream)));
            else
                ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, false>(d_xt[pa], cnt, tri_total, d_state, stream)));
        }
        if (lowp) {
            ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2, true>(d_tab[0][pa][0], cnt, tri_total, d_state, stream)));
            if (root == 4)
                ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2, true>(d_tab[0][pa][1], cnt, tri_total, d_state, stream)));
            ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2, true>(d_tab[0][pa][2], cnt, tri_total, d_state, stream)));
        } else if (p32) {
            ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, false>(d_tab[0][pa][0], cnt, tri_total, d_state, stream)));
            if (root == 4)
                ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, false>(d_tab[0][pa][1], cnt, tri_total, d_state, stream)));
            ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, false>(d_tab[0][pa][2], cnt, tri_total, d_state, stream)));
        } else {
            for (int l = 0; l < 3; ++l) {
                if (l == 1 && root != 4) continue;
                // the M-update of the last fp64 iteration writes the fp32 M the next tier starts from
                const GemmProblem *tab = (l == 2 && k == j64 - 1 && pl.use32) ? d_last64[pa] : d_tab[1][pa][l];
                if (ns8 > 0) {
                    // Cut the A operand into slices, decide per factor, multiply.  T goes to buffer 1
                    // and stays there: T T reads it twice, and T^4 M reads it as M (B mode 1), so M
                    // itself is never cut; T^2 and T^4 go to buffer 0.
                    const dim3 sgrid((unsigned)((i8_rows(n_max) + 3) / 4), (unsigned)cnt);
                    const int abuf = l == 0 ? 1 : 0, bbuf = l == 1 ? 0 : 1, bmode = l == 2 ? 1 : 0;
                    const int lds_k = i8_slice_lds_k(n_max);
                    {   // rows of 1900 to 2048 entries park more than the default 64 KiB of dynamic LDS
                        static bool cfg5s[MAX_DEVICES] = {}, cfg4s[MAX_DEVICES] = {};
                        if (ns8 == 5) ASTERIA_HIP_TRY(ensure_dynamic_lds(reinterpret_cast<const void *>(i8_slice_kernel<5>), i8_slice_lds_bytes(I8_SLICE_LDS_K), cfg5s));
                        else ASTERIA_HIP_TRY(ensure_dynamic_lds(reinterpret_cast<const void *>(i8_slice_kernel<4>), i8_slice_lds_bytes(I8_SLICE_LDS_K), cfg4s));
                    }
                    if (ns8 == 5) hipLaunchKernelGGL(i8_slice_kernel<5>, sgrid, dim3(256), i8_slice_lds_bytes(lds_k), stream, tab, d_xf, d_state, 0, abuf, lds_k);
                    else hipLaunchKernelGGL(i8_slice_kernel<4>, sgrid, dim3(256), i8_slice_lds_bytes(lds_k), stream, tab, d_xf, d_state, 0, abuf, lds_k);
                    // per factor: 4 slices where the estimate allows, else 5 (if the planes have them), else fp64
                    hipLaunchKernelGGL(i8_gate_kernel, dim3(ctl_blocks), dim3(128), 0, stream, d_xf, cnt, &d_fs[0].lo_cur,
                                       (int)sizeof(FactorScal), 4, ns8, abuf, bbuf, bmode,
                                       I8_THETA * 2.0f / (float)std::max(2, j64), d_state, profile_i8_counters());
                    ASTERIA_HIP_TRY(hipGetLastError());
                    if (ns8 == 5) ASTERIA_HIP_TRY((launch_gemm_i8_grouped<5>(tab, d_xf, cnt, tri_total, d_state, abuf, bbuf, bmode, stream)));
                    else ASTERIA_HIP_TRY((launch_gemm_i8_grouped<4>(tab, d_xf, cnt, tri_total, d_state, abuf, bbuf, bmode, stream)));
                }
                ASTERIA_HIP_TRY((launch_gemm_grouped<double, double, double, false, false>(tab, cnt, tri_total, d_state, stream)));
            }
        }
    }
    hipLaunchKernelGGL(root_control_kernel, dim3(cnt), dim3(64), 0, stream, d_fd, d_fs, d_state, K,
                       (K >= j64 && pl.use32) ? 1 : 0, 1, pl.stop_resid, root, pl.adapted ? 1 : 0, pl.xt_lowp ? 1 : 0);
    hipLaunchKernelGGL(root_finalize_kernel, dim3(sq_total), dim3(256), 0, stream, d_fd, d_fs, d_state, cnt,
                       d_sq, first, info, iters, resid, lambda_max);
    ASTERIA_HIP_TRY(hipGetLastError());
    return ASTERIA_OK;
}

}  // namespace

extern "C" asteria_status asteria_inverse_root_plan(int root, asteria_eps_mode mode, const float *eps, int eps_count,
                                                    const asteria_root_opts *opts, int32_t *fp64_iters,
                                                    int32_t *lowp_from, int32_t *x_update_lowp)
{
    if (root != 2 && root != 4) return ASTERIA_UNSUPPORTED;
    if (!eps || eps_count <= 0) return ASTERIA_INVALID_ARG;
    Plan pl;
    const asteria_status st = make_plan(opts, mode, eps, eps_count, root, pl);
    if (st != ASTERIA_OK) return st;
    if (fp64_iters) *fp64_iters = pl.fp64_iters;
    if (lowp_from) *lowp_from = pl.lowp_from;
    if (x_update_lowp) *x_update_lowp = pl.xt_lowp ? 1 : 0;
    return ASTERIA_OK;
}

extern "C" size_t asteria_inverse_root_workspace_bytes(const asteria_factor *f, int nfactors,
                                                       const asteria_root_opts *opts, size_t *min_bytes)
{
    if (min_bytes) *min_bytes = 0;
    if (!f || nfactors <= 0) return 0;
    Plan pl;
    const float e1 = 1e-6f;
    if (make_plan(opts, ASTERIA_EPS_RELATIVE, &e1, 1, 4, pl) != ASTERIA_OK) return 0;
    // sizes must not depend on eps: reserve both precisions unless the caller pinned one
    asteria_root_opts o;
    asteria_root_opts_default(&o);
    if (opts) o = *opts;
    const bool use64 = (o.fp64_iters != 0);
    const bool use32 = !(o.fp64_iters >= o.max_iters && o.fp64_iters > 0);
    size_t total = fixed_bytes(), biggest = 0;
    for (int i = 0; i < nfactors; ++i) {
        if (f[i].n <= 0) return 0;
        const size_t b = factor_matrix_bytes(f[i].n, use64, use32) + factor_small_bytes(f[i].n) +
                         factor_i8_bytes(f[i].n, use64 ? (o.int8_slices < 0 ? 5 : o.int8_slices) : 0);
        total += b;
        biggest = std::max(biggest, b);
    }
    if (min_bytes) *min_bytes = biggest + fixed_bytes();
    return total;
}

extern "C" asteria_status asteria_inverse_root(const asteria_factor *f, int nfactors, int root,
                                               asteria_eps_mode mode, const float *eps, int eps_count,
                                               const asteria_root_opts *opts,
                                               int32_t *info, int32_t *iters, float *resid, float *lambda_max,
                                               void *ws, size_t ws_bytes, void *stream_)
{
    asteria_status st = validate(f, nfactors, root, eps, eps_count);
    if (st != ASTERIA_OK) return st;
    if (mode != ASTERIA_EPS_RELATIVE && mode != ASTERIA_EPS_ABSOLUTE) return ASTERIA_INVALID_ARG;
    Plan pl;
    st = make_plan(opts, mode, eps, eps_count, root, pl);
    if (st != ASTERIA_OK) return st;
    if (!ws) return ASTERIA_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return ASTERIA_INVALID_ARG;   // workspace must be 256-byte aligned
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_);

    // Passes are formed over the caller's order (outputs are indexed by caller position, and a
    // pass covers a contiguous index range), largest pass that fits the workspace.
    std::vector<int> order(nfactors);
    for (int i = 0; i < nfactors; ++i) order[i] = i;
    int first = 0;
    while (first < nfactors) {
        size_t used = fixed_bytes();
        int cnt = 0;
        while (first + cnt < nfactors && cnt < 65535) {   // 65535: y extent of the mat-vec grid
            const int n = f[first + cnt].n;
            const size_t b = factor_matrix_bytes(n, pl.use64, pl.use32) + factor_small_bytes(n) +
                             factor_i8_bytes(n, pl.i8_slices);
            if (used + b > ws_bytes) break;
            used += b;
            ++cnt;
        }
        if (cnt == 0) return ASTERIA_WORKSPACE_TOO_SMALL;
        st = run_pass(f, order, first, cnt, root, mode, eps, eps_count, pl, info, iters, resid, lambda_max,
                      ws, stream, false, nullptr);
        if (st != ASTERIA_OK) return st;
        first += cnt;
    }
    return ASTERIA_OK;
}

// ---- the same call for callers that cannot allocate ---------------------------------------------
// The workspace is a fixed array in the library's device image instead of caller memory.  In host
// code the array's name only stands for the symbol: its device address is looked up once per device
// and that pointer is what the kernels (and nothing else here) receive.
namespace {
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)64 << 20;
constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
static void *g_scratch_ptr[STATIC_SCRATCH_MAX_DEVICES];   // device address of `scratch`, per device

extern "C" size_t asteria_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

extern "C" asteria_status asteria_inverse_root_static(const asteria_factor *f, int nfactors, int root,
                                                      asteria_eps_mode mode, const float *eps, int eps_count,
                                                      const asteria_root_opts *opts,
                                                      int32_t *info, int32_t *iters, float *resid, float *lambda_max,
                                                      void *stream_)
{
    asteria_status st = validate(f, nfactors, root, eps, eps_count);
    if (st != ASTERIA_OK) return st;
    if (mode != ASTERIA_EPS_RELATIVE && mode != ASTERIA_EPS_ABSOLUTE) return ASTERIA_INVALID_ARG;
    Plan pl;
    st = make_plan(opts, mode, eps, eps_count, root, pl);
    if (st != ASTERIA_OK) return st;
    // every factor must fit the array by itself (the call works through the batch in passes)
    for (int i = 0; i < nfactors; ++i) {
        const int n = f[i].n;
        const size_t b = fixed_bytes() + factor_matrix_bytes(n, pl.use64, pl.use32) + factor_small_bytes(n) +
                         factor_i8_bytes(n, pl.i8_slices);
        if (b > STATIC_SCRATCH_BYTES) return ASTERIA_EXCEEDS_STATIC_SCRATCH;
    }
    int dev = -1;
    ASTERIA_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= STATIC_SCRATCH_MAX_DEVICES) return ASTERIA_UNSUPPORTED;
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        ASTERIA_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return ASTERIA_HIP_ERROR;
        g_scratch_ptr[dev] = p;
    }
    return asteria_inverse_root(f, nfactors, root, mode, eps, eps_count, opts, info, iters, resid, lambda_max,
                                g_scratch_ptr[dev], STATIC_SCRATCH_BYTES, stream_);
}
