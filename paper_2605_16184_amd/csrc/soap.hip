// SOAP variant (paper Eq. 2):  N = Q_L phi(Q_L^T G Q_R) Q_R^T with phi = Adam in the rotated
// basis (asteria_soap_step), and the eigenbasis refresh Q <- qr(A Q).Q (asteria_soap_refresh).
//
// soap_step:   four grouped GEMMs (rotate in: G Q_R, then Q_L^T (.); rotate out: N' Q_R^T, then
//              Q_L (.)) around one HBM-streaming Adam kernel, on the bf16 matrix cores with every
//              fp32 operand split into two bf16 terms (16 bits kept, three MFMA passes per product,
//              two when G is bf16): a plain bf16 cast of an eigenbasis costs 0.1-0.5 relative error
//              in N, the split about 1e-5.  That kernel reads k-contiguous operands only, so the
//              call first writes Q_L^T and Q_R^T to the workspace, and the first product of each
//              rotation stores its result transposed.  Blocks whose shapes fill whole 256 x 256
//              tiles run the three split x split products on the 8-wavefront kernel of pgemm.h.
// soap_refresh: Z^T = Q^T A by one grouped GEMM (columns of Z become contiguous rows), then the
//              thin QR factor of Z with diag(R) > 0 - the same Q a Householder QR with that sign
//              convention returns, since the factorisation is unique - by block Gram-Schmidt
//              with re-orthogonalisation: panels of 128 columns; each panel is projected twice
//              against all finished panels (two grouped fp32-MFMA GEMMs per projection, so the
//              O(n^3) work runs on the matrix cores), then orthonormalised by Cholesky QR applied
//              twice: Gram matrix of the panel on the fp64 matrix cores, 128 x 128 Cholesky
//              factor and its inverse in LDS (fp64), panel <- L^-1 panel on the fp32 matrix
//              cores.  The second application removes the cond^2 * 2^-24 loss of the first, so
//              ||Q^T Q - I|| ends at round-off level as long as cond(Z) * 2^-24 < 1, and L's
//              positive diagonal gives the diag(R) > 0 convention.  A transposing write-back
//              stores Q.
#include <algorithm>
#include <vector>

#include "common.h"
#include "gemm.h"
#include "gemm_bf16.h"
#include "pgemm.h"

using namespace asteria;

namespace {

inline int ld4(int n) { return (n + 3) & ~3; }

// ---------------------------------------------------------------------------------------------
// Adam in the rotated basis, elementwise over every block.
struct AdamBlock {
    const float *Gr;   // rotated gradient G' (ld = ldw)
    float *M, *V;      // moments, in place
    float *Np;         // N' out (ld = ldw)
    int m, n, ldw, ldm, ldv;
    int row_start;     // first global row id of this block
};

__global__ __launch_bounds__(256) void adam_rotated_kernel(const AdamBlock *blocks, int nblocks,
                                                           float b1, float b2, float eps,
                                                           float inv_c1, float inv_c2)
{
    // one workgroup per matrix row
    int lo = 0, hi = nblocks - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (blocks[mid].row_start <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
    }
    const AdamBlock &B = blocks[lo];
    const int row = (int)blockIdx.x - B.row_start;
    const float *__restrict__ g = B.Gr + (size_t)row * B.ldw;
    float *__restrict__ mm = B.M + (size_t)row * B.ldm;
    float *__restrict__ vv = B.V + (size_t)row * B.ldv;
    float *__restrict__ np = B.Np + (size_t)row * B.ldw;
    for (int j = threadIdx.x; j < B.n; j += 256) {
        const float gj = g[j];
        const float m1 = b1 * mm[j] + (1.0f - b1) * gj;
        const float v1 = b2 * vv[j] + (1.0f - b2) * gj * gj;
        mm[j] = m1;
        vv[j] = v1;
        np[j] = (m1 * inv_c1) / (sqrtf(v1 * inv_c2) + eps);
    }
}

// ---------------------------------------------------------------------------------------------
// dst = src^T for a batch of fp32 matrices, 32 x 32 tiles through LDS (reads and writes along rows)
struct TransposeF32Job {
    const float *src;   // rows x cols, ld = lds_
    float *dst;         // cols x rows, ld = ldd
    int rows, cols, lds_, ldd;
    int tile_start;
    int pad_;
};

__global__ __launch_bounds__(256) void transpose_f32_kernel(const TransposeF32Job *jobs, int njobs)
{
    int lo = 0, hi = njobs - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (jobs[mid].tile_start <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
    }
    const TransposeF32Job &J = jobs[lo];
    const int lt = (int)blockIdx.x - J.tile_start;
    const int tcols = (J.cols + 31) / 32;
    const int ti = lt / tcols, tj = lt % tcols;
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int rr = ty; rr < 32; rr += 8) {
        const int r = ti * 32 + rr, c = tj * 32 + tx;
        tile[rr][tx] = (r < J.rows && c < J.cols) ? J.src[(size_t)r * J.lds_ + c] : 0.0f;
    }
    __syncthreads();
    for (int rr = ty; rr < 32; rr += 8) {
        const int r = tj * 32 + rr, c = ti * 32 + tx;   // element (r, c) of dst = src(c, r)
        if (r < J.cols && c < J.rows) J.dst[(size_t)r * J.ldd + c] = tile[tx][rr];
    }
}

// ---------------------------------------------------------------------------------------------
// Orthonormalisation of Z^T (row c of Zt = column c of Z), in place.
struct QrFactor {
    float *Zt;      // n x ldz; rows become the orthonormal columns of Q, in order
    float *Qout;    // caller's Q (n x ldq)
    double *gram;   // QR_PANEL x QR_PANEL: Gram matrix of the current panel
    float *winv;    // QR_PANEL x QR_PANEL: inverse Cholesky factor of the current panel
    int n, ldz, ldq;
    int pad0_;
    int bad;        // set to 1 when a column could not be normalised
    // Two words the grouped launches read as their per-problem state (a problem runs while its word
    // is 0): `run` stays 0; `skip3` is 1 unless the second sweep over the current panel found a row
    // that needs a third one.
    int run, skip3;
    int out_index;  // position of this factor in the caller's arrays
    int pad_;
    // Powers of two that bring the rows of the current panel into the fp16 range for the projection
    // coefficients computed on the fp16 cores: a_scale for rows of Z^T as they come out of Q^T A
    // (bounded by tr A), 2^14 once a sweep has normalised them; p_scale is the one in force.
    float a_scale, p_scale;
    const float *A;  // the statistic (read for its trace)
    int lda, pad2_;
    float *cbuf;     // QR_PANEL x ldz: projection coefficients of the current panel
    // Where Q^T stands when a round starts (rows q_i^T: the k-contiguous operand of Z^T = Q^T A): the
    // caller's Q buffer, transposed in place, or a buffer of the caller that holds Q^T beside Q
    float *Qt;
    int ldqt, pad3_;
    double *est;     // n estimated eigenvalues q_i^T A q_i (column order of the refresh's input)
    int *perm;       // n: perm[r] = input column that becomes column r
    int *perm_out;   // the caller's slice of the permutation output, or null
};
constexpr float QR_UNIT_SCALE = 16384.0f;
constexpr int QR_STATE_STRIDE = (int)(sizeof(QrFactor) / sizeof(int));
static_assert(sizeof(QrFactor) % sizeof(int) == 0, "state words are addressed as ints inside the factor array");

// a_scale = p_scale = largest power of two with 2^e tr|A| <= 30000 (|Z_ij| <= ||A||_2 <= tr A for a
// positive semi-definite A and orthonormal Q); one wavefront per factor
__global__ __launch_bounds__(64) void qr_scale_kernel(QrFactor *fs, int nf)
{
    const int f = blockIdx.x;
    if (f >= nf) return;
    const float *a = fs[f].A;
    const int n = fs[f].n, ld = fs[f].lda;
    double t = 0.0;
    for (int i = threadIdx.x; i < n; i += 64) t += fabs((double)a[(size_t)i * ld + i]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) t += __shfl_xor(t, off, 64);
    if (threadIdx.x == 0) {
        int e = (t > 0.0 && t < 1e300) ? (int)floor(log2(30000.0 / t)) : 0;
        e = e < -100 ? -100 : (e > 100 ? 100 : e);
        const float sc = (float)ldexp(1.0, e);
        fs[f].a_scale = sc;
        fs[f].p_scale = sc;
    }
}

constexpr int QR_PANEL = 128;
constexpr int QR_MAXN = 1 << 20;

// One workgroup per (factor, panel).  In: the fp64 Gram matrix G = P P^T of the panel's rows
// (rows x rows, leading dimension QR_PANEL).  Out: W = L^-1 in fp32, where G = L L^T is the
// Cholesky factorisation (positive diagonal), so that W P has orthonormal rows and P = L (W P)
// is the QR relation with a positive diagonal.  Everything runs in LDS in fp64: a right-looking
// Cholesky on a 16 x 16 thread grid, then the triangular inverse in place, row by row (row i of
// W needs row i of L and the rows of W above it; one thread per column).
constexpr int CHOL_THREADS = 256;
// Sweeps and failure reporting.  A pivot that is not positive (a zero row cannot be normalised)
// fails the factor.  In the second sweep over a panel (sweep = 1) the rows are those the first
// sweep normalised, projected once more: a pivot far below 1 there means that a row was
// numerically dependent - the first normalisation blew round-off up to unit length, most of which
// lay in the span of the rows before it - and this sweep's normalisation amplifies what the
// projection left by 1 / sqrt(pivot).  Such a factor takes a third sweep (skip3 = 0), which only
// its workgroups run; a pivot that small in the third sweep fails the factor.
constexpr double CHOL_REPEAT_MIN = 0.1;
constexpr int CHOL_NB = 16;                                   // block size of the factorisation and the inverse
constexpr int CHOL_PITCH = QR_PANEL + 1;
// LDS: the matrix (QR_PANEL x CHOL_PITCH doubles) and a block row of CHOL_NB x QR_PANEL doubles
constexpr size_t CHOL_LDS_BYTES = sizeof(double) * ((size_t)QR_PANEL * CHOL_PITCH + (size_t)CHOL_NB * QR_PANEL);

// Both phases work on blocks of 16 so that the workgroup meets at a barrier a few times per block
// instead of a few times per column: per block column of the Cholesky factorisation one wavefront
// factors the 16 x 16 diagonal block (its lanes stay in step through LDS, which a wavefront accesses in
// order), every row below solves against it, and the trailing matrix takes a rank-16 update; the
// inverse is formed from the inverses of the diagonal blocks, block row by block row.
__global__ __launch_bounds__(CHOL_THREADS) void panel_chol_inverse_kernel(QrFactor *fs, int panel, int sweep)
{
    QrFactor &F = fs[blockIdx.x];                   // the factors that have this panel are the first ones (sorted by size)
    if (sweep == 2 && F.skip3) return;              // uniform over the workgroup
    const int rows = min(QR_PANEL, F.n - panel * QR_PANEL);
    extern __shared__ __align__(16) unsigned char chol_smem[];
    double *L = reinterpret_cast<double *>(chol_smem);            // rows x rows, pitch QR_PANEL + 1
    double *S = L + (size_t)QR_PANEL * CHOL_PITCH;                // CHOL_NB x QR_PANEL
    constexpr int PITCH = CHOL_PITCH;
    constexpr int NB = CHOL_NB;
    __shared__ int bad_flag;
    const int tid = threadIdx.x;
    const int ti = tid >> 4, tj = tid & 15;
    const int lane = tid & 63, wave = tid >> 6;
    if (tid == 0) bad_flag = 0;
    // rows and columns beyond `rows` are those of the identity: the blocks need no edge cases
    for (int i = ti; i < QR_PANEL; i += 16)
        for (int j = tj; j < QR_PANEL; j += 16)
            L[i * PITCH + j] = (i < rows && j < rows) ? F.gram[(size_t)i * QR_PANEL + j] : (i == j ? 1.0 : 0.0);
    __syncthreads();
    const int nblk = (rows + NB - 1) / NB;

    // ---- Cholesky factorisation, lower triangle in place
    for (int kb = 0; kb < nblk; ++kb) {
        const int k0 = kb * NB;
        if (wave == 0) {
            // diagonal block: lane -> elements (i, j) = (e / 16, e % 16), e = lane + 64 q
            for (int k = 0; k < NB; ++k) {
                double piv = L[(k0 + k) * PITCH + k0 + k];
                if (k0 + k < rows) {
                    if (!(piv > 0.0) || !(piv < 1e300)) {        // not positive definite: keep going with a tiny pivot
                        if (lane == 0) bad_flag = 1;
                        piv = 1e-300;
                    } else if (sweep > 0 && piv < CHOL_REPEAT_MIN) {
                        if (lane == 0) bad_flag = 2;
                    }
                }
                const double d = sqrt(piv), rd = 1.0 / d;          // one division per column: the rest multiplies
                if (lane == 0) S[k0 + k] = rd;                     // 1 / L_kk, read by the solves below and by the inverse
                double colv[4], rowv[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int e = lane + 64 * q, i = e >> 4, j = e & 15;
                    colv[q] = L[(k0 + i) * PITCH + k0 + k];      // L[i][k] before scaling
                    rowv[q] = L[(k0 + j) * PITCH + k0 + k];      // L[j][k] before scaling
                }
                __builtin_amdgcn_wave_barrier();                 // all reads of column k precede its rewrite
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int e = lane + 64 * q, i = e >> 4, j = e & 15;
                    if (j == k && i >= k) L[(k0 + i) * PITCH + k0 + k] = (i == k) ? d : colv[q] * rd;
                    else if (j > k && j <= i) L[(k0 + i) * PITCH + k0 + j] -= (colv[q] * rd) * (rowv[q] * rd);
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
        __syncthreads();
        // rows below: L21 = A21 L11^-T, one thread per row
        for (int i = k0 + NB + tid; i < rows; i += CHOL_THREADS) {
            double x[NB];
#pragma unroll
            for (int j = 0; j < NB; ++j) x[j] = L[i * PITCH + k0 + j];
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                double v = x[j];
#pragma unroll
                for (int m = 0; m < j; ++m) v -= x[m] * L[(k0 + j) * PITCH + k0 + m];
                x[j] = v * S[k0 + j];
            }
#pragma unroll
            for (int j = 0; j < NB; ++j) L[i * PITCH + k0 + j] = x[j];
        }
        __syncthreads();
        // trailing matrix: A22 -= L21 L21^T (lower triangle)
        for (int i = k0 + NB + ti; i < rows; i += 16) {
            double li[NB];
#pragma unroll
            for (int m = 0; m < NB; ++m) li[m] = L[i * PITCH + k0 + m];
            for (int j = k0 + NB + tj; j <= i; j += 16) {
                double acc = 0.0;
#pragma unroll
                for (int m = 0; m < NB; ++m) acc += li[m] * L[j * PITCH + k0 + m];
                L[i * PITCH + j] -= acc;
            }
        }
        __syncthreads();
    }

    // ---- W = L^-1 over L.  Diagonal blocks first: lane j of a 16-lane group owns column j of its block.
    {
        const int grp = tid >> 4;                                 // 16 groups of 16 lanes, one block each
        if (grp < nblk) {
            const int k0 = grp * NB, j = tj;
            double w[NB];
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                double sum = (i == j) ? 1.0 : 0.0;
#pragma unroll
                for (int k = 0; k < i; ++k)
                    if (k >= j) sum -= L[(k0 + i) * PITCH + k0 + k] * w[k];
                w[i] = (i >= j) ? sum * S[k0 + i] : 0.0;
            }
            __builtin_amdgcn_wave_barrier();                      // the group's reads of the block precede the rewrite
#pragma unroll
            for (int i = 0; i < NB; ++i)
                if (i >= j) L[(k0 + i) * PITCH + k0 + j] = w[i];
        }
    }
    __syncthreads();
    // Block rows: W_ij = -W_ii (sum_{k = j}^{i - 1} L_ik W_kj), j < i; rows above i already hold W.
    for (int ib = 1; ib < nblk; ++ib) {
        const int i0 = ib * NB;
        // S[ti][c] = sum over k in [c, i0) of L[i0 + ti][k] W[k][c] (W is lower triangular; above its
        // diagonal the array still holds the input), c < i0: thread (ti, tj) takes the columns
        // c = tj, tj + 16, ...
        for (int c = tj; c < i0; c += 16) {
            double acc = 0.0;
            for (int k = c; k < i0; ++k) acc += L[(i0 + ti) * PITCH + k] * L[k * PITCH + c];
            S[ti * QR_PANEL + c] = acc;
        }
        __syncthreads();
        for (int c = tj; c < i0; c += 16) {
            double acc = 0.0;
#pragma unroll
            for (int m = 0; m < NB; ++m)
                if (m <= ti) acc += L[(i0 + ti) * PITCH + i0 + m] * S[m * QR_PANEL + c];   // W_ii is lower triangular
            L[(i0 + ti) * PITCH + c] = -acc;
        }
        __syncthreads();
    }
    for (int i = ti; i < rows; i += 16)
        for (int j = tj; j < rows; j += 16)
            F.winv[(size_t)i * QR_PANEL + j] = (j <= i) ? (float)L[i * PITCH + j] : 0.0f;
    if (tid == 0) {
        if (bad_flag == 1 || (bad_flag == 2 && sweep == 2)) F.bad = 1;
        if (sweep == 0) { F.skip3 = 1; F.p_scale = QR_UNIT_SCALE; }       // the rows are normalised now
        // after the last sweep of a panel the scale goes back to that of the rows of Z^T (the next panel)
        if (sweep == 1) { if (bad_flag == 2) F.skip3 = 0; else F.p_scale = F.a_scale; }
        if (sweep == 2) F.p_scale = F.a_scale;
    }
}

__global__ void qr_info_kernel(const QrFactor *fs, int nf, int32_t *info)
{
    const int f = blockIdx.x * blockDim.x + threadIdx.x;
    if (f < nf && info) info[fs[f].out_index] = fs[f].bad ? ASTERIA_INFO_NOT_PD : ASTERIA_INFO_OK;
}

// Q <- Q^T in place: pairs of mirrored 32 x 32 tiles swapped through LDS.  Grid: x = tile (row-major
// over the largest factor's tile grid; tiles below the diagonal or outside this factor do nothing),
// y = factor.
__global__ __launch_bounds__(256) void transpose_inplace_kernel(const QrFactor *fs)
{
    const QrFactor &F = fs[blockIdx.y];
    if (F.Qt != F.Qout) return;                       // the caller keeps Q^T beside Q: nothing to transpose
    const int tpr = (F.n + 31) / 32, tmax = (int)rintf(sqrtf((float)gridDim.x));
    const int ti = (int)blockIdx.x / tmax, tj = (int)blockIdx.x % tmax;
    if (ti > tj || tj >= tpr) return;
    __shared__ float up[32][33], lo[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int r = ty; r < 32; r += 8) {
        const int i = ti * 32 + r, c = tj * 32 + tx;     // upper tile (ti, tj)
        up[r][tx] = (i < F.n && c < F.n) ? F.Qout[(size_t)i * F.ldq + c] : 0.0f;
        const int i2 = tj * 32 + r, c2 = ti * 32 + tx;   // its mirror (tj, ti)
        lo[r][tx] = (i2 < F.n && c2 < F.n) ? F.Qout[(size_t)i2 * F.ldq + c2] : 0.0f;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int i = ti * 32 + r, c = tj * 32 + tx;
        if (i < F.n && c < F.n) F.Qout[(size_t)i * F.ldq + c] = lo[tx][r];
        const int i2 = tj * 32 + r, c2 = ti * 32 + tx;
        if (ti != tj && i2 < F.n && c2 < F.n) F.Qout[(size_t)i2 * F.ldq + c2] = up[tx][r];
    }
}

// Q[i][c] = Zt[c][i] for the rows c of one finished panel: 32 x 32 tiles through LDS.  Grid:
// x = tile of the 128 x n strip, y = factor (the first ones of the group have the panel).  The caller's Q thus fills up
// panel by panel, and the next panels read the finished columns from it with k contiguous.
__global__ __launch_bounds__(256) void transpose_panel_kernel(const QrFactor *fs, int panel)
{
    const QrFactor &F = fs[blockIdx.y];
    const int tpr = (F.n + 31) / 32;
    const int ti = (int)blockIdx.x / tpr, tj = (int)blockIdx.x % tpr;   // tile row inside the panel, tile column
    const int c0 = panel * QR_PANEL + ti * 32;
    if (ti >= QR_PANEL / 32 || c0 >= F.n) return;
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int r = ty; r < 32; r += 8) {
        const int c = c0 + r, i = tj * 32 + tx;
        tile[r][tx] = (c < F.n && i < F.n) ? F.Zt[(size_t)c * F.ldz + i] : 0.0f;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int i = tj * 32 + r, c = c0 + tx;
        if (i < F.n && c < F.n) F.Qout[(size_t)i * F.ldq + c] = tile[tx][r];
    }
}

// Q = I for every factor of the group (the refresh then starts from the identity)
__global__ __launch_bounds__(256) void set_identity_kernel(const QrFactor *fs)
{
    const QrFactor &F = fs[blockIdx.y];
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < (size_t)F.n * F.n; e += (size_t)gridDim.x * 256) {
        const int i = (int)(e / F.n), j = (int)(e % F.n);
        F.Qout[(size_t)i * F.ldq + j] = (i == j) ? 1.0f : 0.0f;
        if (F.Qt != F.Qout) F.Qt[(size_t)i * F.ldqt + j] = (i == j) ? 1.0f : 0.0f;
    }
}

// Q^T kept beside Q by the caller.  mode 0: Qt <- Q^T (the buffer does not hold it yet), 32 x 32 tiles
// through LDS; mode 1: Qt <- Zt (the rows of Z^T are the new basis vectors when a round ends), a plain
// copy.  Grid: x = 32 x 32 tile of the largest factor's tile grid, y = factor; factors without such a
// buffer do nothing.
__global__ __launch_bounds__(256) void keep_qt_kernel(const QrFactor *fs, int mode)
{
    const QrFactor &F = fs[blockIdx.y];
    if (F.Qt == F.Qout) return;
    const int tpr = (F.n + 31) / 32, tmax = (int)rintf(sqrtf((float)gridDim.x));
    const int ti = (int)blockIdx.x / tmax, tj = (int)blockIdx.x % tmax;
    if (ti >= tpr || tj >= tpr) return;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    if (mode == 1) {
        // one 16-byte piece per thread where the caller's buffer allows it (the workspace rows always do)
        const bool vec = ((reinterpret_cast<uintptr_t>(F.Qt) & 15u) == 0) && ((F.ldqt & 3) == 0);
        const int i = ti * 32 + (int)(threadIdx.x >> 3), c = tj * 32 + 4 * (int)(threadIdx.x & 7);
        if (i >= F.n || c >= F.n) return;
        const float *src = F.Zt + (size_t)i * F.ldz + c;
        float *dst = F.Qt + (size_t)i * F.ldqt + c;
        if (vec && c + 4 <= F.n) {
            *reinterpret_cast<float4 *>(dst) = *reinterpret_cast<const float4 *>(src);
        } else {
            for (int e = 0; e < 4 && c + e < F.n; ++e) dst[e] = src[e];
        }
        return;
    }
    __shared__ float tile[32][33];
    for (int r = ty; r < 32; r += 8) {
        const int i = ti * 32 + r, c = tj * 32 + tx;
        tile[r][tx] = (i < F.n && c < F.n) ? F.Qout[(size_t)i * F.ldq + c] : 0.0f;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int i = tj * 32 + r, c = ti * 32 + tx;     // Qt(i, c) = Q(c, i)
        if (i < F.n && c < F.n) F.Qt[(size_t)i * F.ldqt + c] = tile[tx][r];
    }
}

// Column order of the basis before the refresh (the order SOAP uses): est_i = q_i^T A q_i, largest
// first, ties by index.  With Q^T in the caller's buffer (rows q_i^T) and Z^T = Q^T A already formed,
// est_i is the dot product of row i of the two; one wavefront per row, fp64 sums.
__global__ __launch_bounds__(256) void sort_estimate_kernel(const QrFactor *fs)
{
    const QrFactor &F = fs[blockIdx.y];
    const int row = (int)blockIdx.x * 4 + (int)(threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= F.n) return;
    const float *q = F.Qt + (size_t)row * F.ldqt, *z = F.Zt + (size_t)row * F.ldz;
    double s = 0.0;
    for (int k = lane; k < F.n; k += 64) s += (double)q[k] * (double)z[k];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) F.est[row] = s;
}

// rank of every estimate: the number of columns that come before it (larger estimate, or equal and a
// lower index); perm[rank] = column.  n comparisons per column: cheap next to the products.
__global__ __launch_bounds__(256) void sort_rank_kernel(const QrFactor *fs)
{
    const QrFactor &F = fs[blockIdx.y];
    const int i = (int)blockIdx.x * 256 + threadIdx.x;
    __shared__ double chunk[256];
    const double mine = i < F.n ? F.est[i] : 0.0;
    int rank = 0;
    for (int j0 = 0; j0 < F.n; j0 += 256) {
        __syncthreads();
        chunk[threadIdx.x] = j0 + (int)threadIdx.x < F.n ? F.est[j0 + threadIdx.x] : 0.0;
        __syncthreads();
        const int lim = min(256, F.n - j0);
        for (int t = 0; t < lim; ++t) {
            const double o = chunk[t];
            rank += (o > mine || (o == mine && j0 + t < i)) ? 1 : 0;
        }
    }
    if (i < F.n) {
        F.perm[rank] = i;
        if (F.perm_out) F.perm_out[rank] = i;
    }
}

// rows of Z^T gathered in the new order, through the caller's Q buffer (free between the product that
// formed Z^T and the first finished panel): phase 0: Q[r] = Zt[perm[r]]; phase 1: Zt[r] = Q[r]
__global__ __launch_bounds__(256) void sort_gather_kernel(const QrFactor *fs, int phase)
{
    const QrFactor &F = fs[blockIdx.y];
    const int row = (int)blockIdx.x;
    if (row >= F.n) return;
    const float *src = phase == 0 ? F.Zt + (size_t)F.perm[row] * F.ldz : F.Qout + (size_t)row * F.ldq;
    float *dst = phase == 0 ? F.Qout + (size_t)row * F.ldq : F.Zt + (size_t)row * F.ldz;
    for (int k = threadIdx.x; k < F.n; k += 256) dst[k] = src[k];
}

// Problem tables of one group of factors, written on the device from the factor descriptors (as host
// tables they travel as kernel arguments: about 500 upload launches per group of the 1B-model workload).
// The factors of a group are sorted by size, largest first, so those that have panel j are the first
// count_j of the group and the entry of factor i in any table of panel j is entry i of that panel's run.
struct RefreshTables {
    GemmProblem *z;                    // Z^T = Q^T A: one entry per factor
    GemmProblem *t1, *t2, *t3, *t4;    // projection coefficients, projection, Gram matrix, application of L^-1
    const int *off;                    // np + 1: start of panel j's run in t1 .. t4
    const int *pt;                     // cnt + 1: tile columns (ceil(n / 128)) of the factors before i
    const int *pz;                     // cnt + 1: tiles of the Z product (ceil(n / 128)^2) of the factors before i
};

__global__ __launch_bounds__(128) void refresh_tables_kernel(QrFactor *fs, int cnt, RefreshTables T)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x, j = blockIdx.y;
    if (i >= cnt) return;
    const QrFactor F = fs[i];
    const float *a_scale = &fs[i].a_scale, *p_scale = &fs[i].p_scale;
    const int tn = (F.n + BN - 1) / BN;
    GemmProblem p = {};
    p.alpha = 1.0f; p.beta = 0.0f;
    if (j == 0) {
        // Z^T = Q^T A on the fp16 cores (two terms per operand): A'(i, k) = Q^T[i][k] - the caller's Q has
        // been transposed in place by then, or the caller keeps Q^T -, scaled by 2^14, and B'(j, k) = A[j][k] (A is symmetric),
        // scaled by the factor's a_scale; both k-contiguous
        GemmProblem g = p;
        g.state_idx = -1; g.state_mask = ~0;
        g.M = g.N = g.K = F.n; g.tiles_n = tn;
        g.A = F.Qt; g.lda = F.ldqt; g.B = F.A; g.ldb = F.lda; g.C = F.Zt; g.ldc = F.ldz;
        g.sa = QR_UNIT_SCALE; g.sb_dev = a_scale;
        g.tile_start = T.pz[i];
        T.z[i] = g;
    }
    if (F.n <= j * QR_PANEL) return;
    const int e = T.off[j] + i;
    const int rows = min(QR_PANEL, F.n - j * QR_PANEL), done = j * QR_PANEL;
    float *Pt = F.Zt + (size_t)done * F.ldz;
    // runs while the factor's state word (`run`, or `skip3` in the third sweep) is 0
    p.state_idx = i * QR_STATE_STRIDE; p.state_mask = 1;
    // Gram matrix of the panel rows (fp64 accumulation), one symmetric tile
    p.flags = GEMM_SYM;
    p.M = rows; p.N = rows; p.K = F.n;
    p.A = Pt; p.lda = F.ldz; p.B = Pt; p.ldb = F.ldz; p.C = F.gram; p.ldc = QR_PANEL;
    p.tile_start = i;
    T.t3[e] = p;
    // P <- W P, in place: the single tile row reads a column range of P completely before it stores
    // the same range
    p.flags = 0;
    p.M = rows; p.N = F.n; p.K = rows; p.tiles_n = tn;
    p.A = F.winv; p.lda = QR_PANEL; p.B = Pt; p.ldb = F.ldz; p.C = Pt; p.ldc = F.ldz;
    p.tile_start = T.pt[i];
    T.t4[e] = p;
    if (j == 0) return;
    // C = P Q_done^T: rows of the panel against the finished rows, contraction over n; on the fp16 cores
    // the panel rows are scaled by the factor's p_scale, the finished rows are orthonormal
    p.M = rows; p.N = done; p.K = F.n; p.tiles_n = j;
    p.A = Pt; p.lda = F.ldz; p.B = F.Zt; p.ldb = F.ldz; p.C = F.cbuf; p.ldc = F.ldz;
    p.tile_start = i * j;                      // every factor of the run has j tile columns here
    p.sa_dev = p_scale; p.sb = QR_UNIT_SCALE;
    T.t1[e] = p;
    // P <- P - C Q_done: contraction over the finished rows, which the caller's Q already holds as
    // columns (k contiguous); the coefficients share the scale of the panel rows
    p.alpha = -1.0f; p.beta = 1.0f;
    p.M = rows; p.N = F.n; p.K = done; p.tiles_n = tn;
    p.A = F.cbuf; p.lda = F.ldz; p.B = F.Qout; p.ldb = F.ldq; p.C = Pt; p.ldc = F.ldz;
    p.tile_start = T.pt[i];
    T.t2[e] = p;
}

asteria_status validate_step(const asteria_sblock *b, int nblocks, float b1, float b2, float eps, int t)
{
    if (!b || nblocks <= 0 || t < 1) return ASTERIA_INVALID_ARG;
    if (!(b1 >= 0.0f && b1 < 1.0f) || !(b2 >= 0.0f && b2 < 1.0f) || !(eps >= 0.0f)) return ASTERIA_INVALID_ARG;
    for (int i = 0; i < nblocks; ++i) {
        const asteria_sblock &k = b[i];
        if (!k.G || (!k.QL && !k.QR) || !k.M || !k.V || !k.N) return ASTERIA_INVALID_ARG;   // one side may be the identity
        if (k.m <= 0 || k.n <= 0) return ASTERIA_INVALID_ARG;
        if (k.ldg < k.n || (k.QL && k.ldql < k.m) || (k.QR && k.ldqr < k.n) || k.ldm < k.n || k.ldv < k.n || k.ldn < k.n)
            return ASTERIA_INVALID_ARG;
        if (!valid_dtype(k.g_dtype)) return ASTERIA_INVALID_ARG;
        if ((k.QLt && k.ldqlt < k.m) || (k.QRt && k.ldqrt < k.n)) return ASTERIA_INVALID_ARG;
    }
    return ASTERIA_OK;
}

// The same transposition for descriptors that travel as kernel arguments (asteria_transpose has no workspace).
constexpr int TRANSPOSE_CHUNK = 64;
struct TransposeChunk {
    TransposeF32Job job[TRANSPOSE_CHUNK];
};

__global__ __launch_bounds__(256) void transpose_chunk_kernel(TransposeChunk c, int njobs)
{
    int lo = 0, hi = njobs - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (c.job[mid].tile_start <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
    }
    const TransposeF32Job &J = c.job[lo];
    const int lt = (int)blockIdx.x - J.tile_start;
    const int tcols = (J.cols + 31) / 32;
    const int ti = lt / tcols, tj = lt % tcols;
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int rr = ty; rr < 32; rr += 8) {
        const int r = ti * 32 + rr, cc = tj * 32 + tx;
        tile[rr][tx] = (r < J.rows && cc < J.cols) ? J.src[(size_t)r * J.lds_ + cc] : 0.0f;
    }
    __syncthreads();
    for (int rr = ty; rr < 32; rr += 8) {
        const int r = tj * 32 + rr, cc = ti * 32 + tx;   // element (r, cc) of dst = src(cc, r)
        if (r < J.cols && cc < J.rows) J.dst[(size_t)r * J.ldd + cc] = tile[tx][rr];
    }
}

}  // namespace

extern "C" asteria_status asteria_transpose(const asteria_tpair *items, int nitems, void *stream_)
{
    if (!items || nitems <= 0) return ASTERIA_INVALID_ARG;
    for (int i = 0; i < nitems; ++i) {
        const asteria_tpair &t = items[i];
        if (!t.src || !t.dst || t.rows <= 0 || t.cols <= 0 || t.lds < t.cols || t.ldd < t.rows) return ASTERIA_INVALID_ARG;
    }
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_);
    for (int first = 0; first < nitems; first += TRANSPOSE_CHUNK) {
        const int cnt = std::min(TRANSPOSE_CHUNK, nitems - first);
        TransposeChunk c;
        memset(&c, 0, sizeof(c));
        int tiles = 0;
        for (int i = 0; i < cnt; ++i) {
            const asteria_tpair &t = items[first + i];
            TransposeF32Job &J = c.job[i];
            J.src = t.src; J.dst = t.dst; J.rows = t.rows; J.cols = t.cols; J.lds_ = t.lds; J.ldd = t.ldd;
            J.tile_start = tiles;
            tiles += ((t.rows + 31) / 32) * ((t.cols + 31) / 32);
        }
        hipLaunchKernelGGL(transpose_chunk_kernel, dim3(tiles), dim3(256), 0, stream, c, cnt);
        ASTERIA_HIP_TRY(hipGetLastError());
    }
    return ASTERIA_OK;
}

extern "C" size_t asteria_soap_step_workspace_bytes(const asteria_sblock *blocks, int nblocks)
{
    if (!blocks || nblocks <= 0) return 0;
    size_t bytes = 4 * Carver::need((size_t)nblocks, sizeof(GemmProblem)) + Carver::need((size_t)nblocks, sizeof(AdamBlock)) +
                   Carver::need(2 * (size_t)nblocks, sizeof(TransposeF32Job)) +
                   3 * Carver::need((size_t)nblocks, sizeof(PlaneProblem)) + Carver::need(4 * (size_t)nblocks, sizeof(GemmProblem)) + 2048;
    for (int i = 0; i < nblocks; ++i) {
        const int m = blocks[i].m, n = blocks[i].n;
        bytes += 2 * Carver::need((size_t)m * ld4(n), sizeof(float));      // G' / N' (m x n)
        bytes += Carver::need((size_t)n * ld4(m), sizeof(float));          // transposed intermediate (n x m)
        if (!blocks[i].QLt) bytes += Carver::need((size_t)m * ld4(m), sizeof(float));   // Q_L^T, unless the caller keeps it
        if (!blocks[i].QRt) bytes += Carver::need((size_t)n * ld4(n), sizeof(float));   // Q_R^T
    }
    return bytes;
}

extern "C" asteria_status asteria_soap_step(const asteria_sblock *blocks, int nblocks,
                                            float beta1, float beta2, float adam_eps, int step_t,
                                            void *ws, size_t ws_bytes, void *stream_)
{
    asteria_status st = validate_step(blocks, nblocks, beta1, beta2, adam_eps, step_t);
    if (st != ASTERIA_OK) return st;
    if (!ws || ws_bytes < asteria_soap_step_workspace_bytes(blocks, nblocks)) return ASTERIA_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return ASTERIA_INVALID_ARG;   // workspace must be 256-byte aligned
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_);

    Carver cv(ws);
    GemmProblem *d_g[4];
    for (int i = 0; i < 4; ++i) d_g[i] = cv.take<GemmProblem>(nblocks);
    AdamBlock *d_ab = cv.take<AdamBlock>(nblocks);
    TransposeF32Job *d_tj = cv.take<TransposeF32Job>(2 * (size_t)nblocks);
    PlaneProblem *d_f[3];
    for (int i = 0; i < 3; ++i) d_f[i] = cv.take<PlaneProblem>(nblocks);
    std::vector<PlaneProblem> f2, f3, f4;   // products 2-4 of blocks that fill whole 256 x 256 tiles
    int tilesf = 0;
    std::vector<GemmProblem> g1[2], g2, g3, g4;
    // one-sided blocks (Q_L or Q_R absent = the identity on that side, e.g. a dimension above the
    // preconditioner cap): one product per rotation, on the fp32 matrix cores, operands read in place
    std::vector<GemmProblem> oL1[2], oL2, oR1[2], oR2;     // left only: Q_L^T G, Q_L N';  right only: G Q_R, N' Q_R^T
    int tL1[2] = {0, 0}, tL2 = 0, tR1[2] = {0, 0}, tR2 = 0;
    std::vector<AdamBlock> ab;
    std::vector<TransposeF32Job> tj;
    int tiles1[2] = {0, 0}, tiles = 0, tilesT = 0, rows = 0, ttiles = 0;
    for (int i = 0; i < nblocks; ++i) {
        const asteria_sblock &k = blocks[i];
        const int ldw = ld4(k.n), ldt = ld4(k.m);
        const int ldqlt = k.QLt ? k.ldqlt : ld4(k.m), ldqrt = k.QRt ? k.ldqrt : ld4(k.n);
        float *Gr = cv.take<float>((size_t)k.m * ldw);   // G' (m x n)
        float *Np = cv.take<float>((size_t)k.m * ldw);   // N' (m x n)
        if (!k.QL || !k.QR) {
            const int tm1 = (k.m + BM - 1) / BM, tn1 = (k.n + BN - 1) / BN;
            GemmProblem p;
            memset(&p, 0, sizeof(p));
            p.state_idx = -1; p.state_mask = ~0; p.alpha = 1.0f; p.beta = 0.0f;
            p.M = k.m; p.N = k.n; p.tiles_n = tn1;
            if (k.QL) {
                // G' = Q_L^T G: A'(i, l) = Q_L[l][i], B'(j, l) = G[l][j], both k-major
                p.K = k.m; p.A = k.QL; p.lda = k.ldql; p.B = k.G; p.ldb = k.ldg; p.C = Gr; p.ldc = ldw;
                p.tile_start = tL1[k.g_dtype]; tL1[k.g_dtype] += tm1 * tn1;
                oL1[k.g_dtype].push_back(p);
                // N = Q_L N': A'(i, l) = Q_L[i][l], B'(j, l) = N'[l][j] (k-major)
                p.A = k.QL; p.lda = k.ldql; p.B = Np; p.ldb = ldw; p.C = k.N; p.ldc = k.ldn;
                p.tile_start = tL2; tL2 += tm1 * tn1;
                oL2.push_back(p);
            } else {
                // G' = G Q_R: A' = G, B'(j, l) = Q_R[l][j] (k-major)
                p.K = k.n; p.A = k.G; p.lda = k.ldg; p.B = k.QR; p.ldb = k.ldqr; p.C = Gr; p.ldc = ldw;
                p.tile_start = tR1[k.g_dtype]; tR1[k.g_dtype] += tm1 * tn1;
                oR1[k.g_dtype].push_back(p);
                // N = N' Q_R^T: A' = N', B'(j, l) = Q_R[j][l]
                p.A = Np; p.lda = ldw; p.B = k.QR; p.ldb = k.ldqr; p.C = k.N; p.ldc = k.ldn;
                p.tile_start = tR2; tR2 += tm1 * tn1;
                oR2.push_back(p);
            }
            AdamBlock a1;
            a1.Gr = Gr; a1.M = k.M; a1.V = k.V; a1.Np = Np; a1.m = k.m; a1.n = k.n; a1.ldw = ldw; a1.ldm = k.ldm; a1.ldv = k.ldv;
            a1.row_start = rows; rows += k.m;
            ab.push_back(a1);
            continue;
        }
        float *Tt = cv.take<float>((size_t)k.n * ldt);   // (G Q_R)^T, later (N' Q_R^T)^T  (n x m)
        // transposed bases: the caller's copies, or made here
        const float *QLt = k.QLt, *QRt = k.QRt;
        TransposeF32Job t;
        memset(&t, 0, sizeof(t));
        if (!QLt) {
            float *dst = cv.take<float>((size_t)k.m * ldqlt);
            t.src = k.QL; t.dst = dst; t.rows = k.m; t.cols = k.m; t.lds_ = k.ldql; t.ldd = ldqlt;
            t.tile_start = ttiles; ttiles += ((k.m + 31) / 32) * ((k.m + 31) / 32);
            tj.push_back(t);
            QLt = dst;
        }
        if (!QRt) {
            float *dst = cv.take<float>((size_t)k.n * ldqrt);
            t.src = k.QR; t.dst = dst; t.rows = k.n; t.cols = k.n; t.lds_ = k.ldqr; t.ldd = ldqrt;
            t.tile_start = ttiles; ttiles += ((k.n + 31) / 32) * ((k.n + 31) / 32);
            tj.push_back(t);
            QRt = dst;
        }
        const int tm = (k.m + BM - 1) / BM, tn = (k.n + BN - 1) / BN;
        GemmProblem p;
        memset(&p, 0, sizeof(p));
        p.state_idx = -1; p.state_mask = ~0; p.alpha = 1.0f; p.beta = 0.0f;
        // 1: (G Q_R)^T:   A' = G (m x n), B' = Q_R^T (B'(j, k) = Q_R[k][j]); m x n result stored transposed
        p.M = k.m; p.N = k.n; p.K = k.n; p.tiles_n = tn;
        p.A = k.G; p.lda = k.ldg; p.B = QRt; p.ldb = ldqrt; p.C = Tt; p.ldc = ldt; p.flags = GEMM_STORE_T;
        p.tile_start = tiles1[k.g_dtype]; tiles1[k.g_dtype] += tm * tn;
        g1[k.g_dtype].push_back(p);
        const bool fast = pg_f32_operand_ok(QLt, k.m, k.m, ldqlt) && pg_f32_operand_ok(Tt, k.n, k.m, ldt) &&
                          pg_f32_operand_ok(Np, k.m, k.n, ldw) && pg_f32_operand_ok(k.QR, k.n, k.n, k.ldqr) &&
                          pg_f32_operand_ok(k.QL, k.m, k.m, k.ldql);
        if (fast) {
            PlaneProblem q;
            memset(&q, 0, sizeof(q));
            q.M = k.m; q.N = k.n; q.tiles_n = k.n / PgF32x2::TN; q.tile_start = tilesf;
            q.state_idx = -1; q.state_mask = ~0; q.alpha = 1.0f; q.beta = 0.0f;
            q.K = k.m; q.A = QLt; q.lda = ldqlt; q.B = Tt; q.ldb = ldt; q.C32 = Gr; q.ldc32 = ldw; q.flags = 0;
            f2.push_back(q);
            q.K = k.n; q.A = Np; q.lda = ldw; q.B = k.QR; q.ldb = k.ldqr; q.C32 = Tt; q.ldc32 = ldt; q.flags = GEMM_STORE_T;
            f3.push_back(q);
            q.K = k.m; q.A = k.QL; q.lda = k.ldql; q.B = Tt; q.ldb = ldt; q.C32 = k.N; q.ldc32 = k.ldn; q.flags = 0;
            f4.push_back(q);
            tilesf += (k.m / PgF32x2::TM) * q.tiles_n;
        } else {
            // 2: G' = Q_L^T (G Q_R):   A' = Q_L^T (m x m), B' = (G Q_R)^T (n x m)
            p.K = k.m; p.A = QLt; p.lda = ldqlt; p.B = Tt; p.ldb = ldt; p.C = Gr; p.ldc = ldw; p.flags = 0;
            p.tile_start = tiles;
            g2.push_back(p);
            // 3: (N' Q_R^T)^T:   A' = N' (m x n), B' = Q_R (B'(j, k) = Q_R[j][k]); stored transposed
            p.K = k.n; p.A = Np; p.lda = ldw; p.B = k.QR; p.ldb = k.ldqr; p.C = Tt; p.ldc = ldt; p.flags = GEMM_STORE_T;
            g3.push_back(p);
            // 4: N = Q_L (N' Q_R^T):   A' = Q_L (m x m), B' = (N' Q_R^T)^T (n x m)
            p.K = k.m; p.A = k.QL; p.lda = k.ldql; p.B = Tt; p.ldb = ldt; p.C = k.N; p.ldc = k.ldn; p.flags = 0;
            g4.push_back(p);
            tiles += tm * tn;
        }
        AdamBlock a;
        a.Gr = Gr; a.M = k.M; a.V = k.V; a.Np = Np; a.m = k.m; a.n = k.n; a.ldw = ldw; a.ldm = k.ldm; a.ldv = k.ldv;
        a.row_start = rows; rows += k.m;
        ab.push_back(a);
    }
    (void)tilesT;
    GemmProblem *d_g1b = d_g[0] + g1[0].size();
    if (!g1[0].empty()) ASTERIA_HIP_TRY(upload_async(d_g[0], g1[0].data(), g1[0].size() * sizeof(GemmProblem), stream));
    if (!g1[1].empty()) ASTERIA_HIP_TRY(upload_async(d_g1b, g1[1].data(), g1[1].size() * sizeof(GemmProblem), stream));
    if (!g2.empty()) {
        ASTERIA_HIP_TRY(upload_async(d_g[1], g2.data(), g2.size() * sizeof(GemmProblem), stream));
        ASTERIA_HIP_TRY(upload_async(d_g[2], g3.data(), g3.size() * sizeof(GemmProblem), stream));
        ASTERIA_HIP_TRY(upload_async(d_g[3], g4.data(), g4.size() * sizeof(GemmProblem), stream));
    }
    if (!f2.empty()) {
        ASTERIA_HIP_TRY(upload_async(d_f[0], f2.data(), f2.size() * sizeof(PlaneProblem), stream));
        ASTERIA_HIP_TRY(upload_async(d_f[1], f3.data(), f3.size() * sizeof(PlaneProblem), stream));
        ASTERIA_HIP_TRY(upload_async(d_f[2], f4.data(), f4.size() * sizeof(PlaneProblem), stream));
    }
    ASTERIA_HIP_TRY(upload_async(d_ab, ab.data(), ab.size() * sizeof(AdamBlock), stream));
    // tables of the one-sided blocks, one after the other in a region of their own
    GemmProblem *d_o = cv.take<GemmProblem>(4 * (size_t)nblocks);
    GemmProblem *d_oL1[2], *d_oR1[2], *d_oL2, *d_oR2;
    {
        GemmProblem *q = d_o;
        auto put = [&](const std::vector<GemmProblem> &v, GemmProblem *&dst) -> hipError_t {
            dst = q;
            q += v.size();
            return v.empty() ? hipSuccess : upload_async(dst, v.data(), v.size() * sizeof(GemmProblem), stream);
        };
        ASTERIA_HIP_TRY(put(oL1[0], d_oL1[0])); ASTERIA_HIP_TRY(put(oL1[1], d_oL1[1])); ASTERIA_HIP_TRY(put(oL2, d_oL2));
        ASTERIA_HIP_TRY(put(oR1[0], d_oR1[0])); ASTERIA_HIP_TRY(put(oR1[1], d_oR1[1])); ASTERIA_HIP_TRY(put(oR2, d_oR2));
    }
    if (!tj.empty()) {
        ASTERIA_HIP_TRY(upload_async(d_tj, tj.data(), tj.size() * sizeof(TransposeF32Job), stream));
        hipLaunchKernelGGL(transpose_f32_kernel, dim3(ttiles), dim3(256), 0, stream, d_tj, (int)tj.size());
        ASTERIA_HIP_TRY(hipGetLastError());
    }
    // one-sided rotations into the eigenbasis
    ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, true, true>(d_oL1[0], (int)oL1[0].size(), tL1[0], nullptr, stream)));
    ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, bf16_t, true, true>(d_oL1[1], (int)oL1[1].size(), tL1[1], nullptr, stream)));
    ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, true>(d_oR1[0], (int)oR1[0].size(), tR1[0], nullptr, stream)));
    ASTERIA_HIP_TRY((launch_gemm_grouped<float, bf16_t, float, false, true>(d_oR1[1], (int)oR1[1].size(), tR1[1], nullptr, stream)));
    if (!g1[0].empty())
        ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2>(d_g[0], (int)g1[0].size(), tiles1[0], nullptr, stream)));
    if (!g1[1].empty())
        ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<bf16_t, float, 1, 2>(d_g1b, (int)g1[1].size(), tiles1[1], nullptr, stream)));
    if (!g2.empty()) ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2>(d_g[1], (int)g2.size(), tiles, nullptr, stream)));
    if (!f2.empty()) ASTERIA_HIP_TRY((launch_pgemm<PgF32x2>(d_f[0], (int)f2.size(), tilesf, nullptr, stream, 513)));
    const float c1 = 1.0f - powf(beta1, (float)step_t), c2 = 1.0f - powf(beta2, (float)step_t);
    hipLaunchKernelGGL(adam_rotated_kernel, dim3(rows), dim3(256), 0, stream, d_ab, nblocks, beta1, beta2,
                       adam_eps, 1.0f / c1, 1.0f / c2);
    ASTERIA_HIP_TRY(hipGetLastError());
    if (!g2.empty()) ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2>(d_g[2], (int)g3.size(), tiles, nullptr, stream)));
    if (!f2.empty()) ASTERIA_HIP_TRY((launch_pgemm<PgF32x2>(d_f[1], (int)f3.size(), tilesf, nullptr, stream, 513)));
    if (!g2.empty()) ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2>(d_g[3], (int)g4.size(), tiles, nullptr, stream)));
    if (!f2.empty()) ASTERIA_HIP_TRY((launch_pgemm<PgF32x2>(d_f[2], (int)f4.size(), tilesf, nullptr, stream, 513)));
    // one-sided rotations back
    ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, true>(d_oL2, (int)oL2.size(), tL2, nullptr, stream)));
    ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, false>(d_oR2, (int)oR2.size(), tR2, nullptr, stream)));
    return ASTERIA_OK;
}

namespace {

size_t refresh_factor_bytes(int n)
{
    const int np = (n + QR_PANEL - 1) / QR_PANEL;
    return Carver::need((size_t)n * ld4(n), sizeof(float)) +            // Z^T, becomes Q^T
           Carver::need((size_t)QR_PANEL * ld4(n), sizeof(float)) +     // projection coefficients of one panel
           Carver::need((size_t)QR_PANEL * QR_PANEL, sizeof(double)) +  // panel Gram matrix / fp64 inverse factor
           Carver::need((size_t)QR_PANEL * QR_PANEL, sizeof(float)) +   // fp32 inverse factor
           Carver::need((size_t)n, sizeof(double)) + Carver::need((size_t)n, sizeof(int)) +   // column estimates and order
           (size_t)(1 + 4 * np) * sizeof(GemmProblem) + (size_t)(np + 2) * sizeof(int) + sizeof(QrFactor);
}

// The factors of a call can be dealt to up to this many groups, each enqueued as a whole on an
// auxiliary stream the caller supplies (asteria_soap_refresh_overlapped); 4 groups: 328 ms against 318
// for 2 on the 1B-model workload (every group brings its own chain of launches).
constexpr int REFRESH_MAX_GROUPS = 4;

size_t refresh_fixed_bytes(int n_max)
{
    const int np = (n_max + QR_PANEL - 1) / QR_PANEL;
    return REFRESH_MAX_GROUPS * ((size_t)(5 * np + 4) * 256 + 4096);   // alignment slack of the per-panel tables, per group
}

}  // namespace

extern "C" size_t asteria_soap_refresh_workspace_bytes(const asteria_factor *f, int nfactors, size_t *min_bytes)
{
    if (min_bytes) *min_bytes = 0;
    if (!f || nfactors <= 0) return 0;
    size_t total = 0, biggest = 0;
    int n_max = 0;
    for (int i = 0; i < nfactors; ++i) {
        const int n = f[i].n;
        if (n <= 0) return 0;
        const size_t b = refresh_factor_bytes(n);
        total += b;
        biggest = b > biggest ? b : biggest;
        n_max = n > n_max ? n : n_max;
    }
    if (min_bytes) *min_bytes = biggest + refresh_fixed_bytes(n_max);
    return total + refresh_fixed_bytes(n_max);
}

extern "C" asteria_status asteria_soap_refresh(const asteria_factor *f, int nfactors, int32_t *info,
                                               void *ws, size_t ws_bytes, void *stream_)
{
    return asteria_soap_refresh_ex(f, nfactors, nullptr, info, nullptr, ws, ws_bytes, stream_);
}

extern "C" void asteria_soap_refresh_opts_default(asteria_soap_refresh_opts *o)
{
    if (!o) return;
    o->sort = 0; o->from_identity = 0; o->rounds = 1; o->n_aux = 0; o->aux_streams = nullptr;
    o->Xt = nullptr; o->ldxt = nullptr; o->xt_in = 0;
}

extern "C" asteria_status asteria_soap_refresh_ex(const asteria_factor *f, int nfactors,
                                                  const asteria_soap_refresh_opts *opts_in, int32_t *info, int32_t *perm,
                                                  void *ws, size_t ws_bytes, void *stream_)
{
    if (!f || nfactors <= 0) return ASTERIA_INVALID_ARG;
    asteria_soap_refresh_opts o;
    asteria_soap_refresh_opts_default(&o);
    if (opts_in) o = *opts_in;
    if ((o.sort != 0 && o.sort != 1) || (o.from_identity != 0 && o.from_identity != 1) || o.rounds < 1 || o.rounds > 1000)
        return ASTERIA_INVALID_ARG;
    if (perm && (!o.sort || o.rounds != 1)) return ASTERIA_INVALID_ARG;   // the order of ONE sorted round can be reported
    if (o.xt_in != 0 && o.xt_in != 1) return ASTERIA_INVALID_ARG;
    if ((o.Xt != nullptr) != (o.ldxt != nullptr)) return ASTERIA_INVALID_ARG;
    void *const *aux_streams = o.aux_streams;
    const int n_aux = o.n_aux;
    if (n_aux < 0 || n_aux > REFRESH_MAX_GROUPS || (n_aux > 0 && !aux_streams)) return ASTERIA_INVALID_ARG;
    for (int g = 0; g < n_aux; ++g)
        if (!aux_streams[g] || aux_streams[g] == stream_) return ASTERIA_INVALID_ARG;
    int n_all = 0;
    for (int i = 0; i < nfactors; ++i) {
        if (!f[i].A || !f[i].X || f[i].n <= 0 || f[i].lda < f[i].n || f[i].ldx < f[i].n) return ASTERIA_INVALID_ARG;
        if (f[i].a_layout != ASTERIA_LAYOUT_FULL) return ASTERIA_UNSUPPORTED;   // A is an operand of the product A Q: full storage
        if (f[i].n > QR_MAXN) return ASTERIA_UNSUPPORTED;
        if (o.Xt && o.Xt[i] && (o.ldxt[i] < f[i].n || o.Xt[i] == f[i].X)) return ASTERIA_INVALID_ARG;
        n_all = f[i].n > n_all ? f[i].n : n_all;
    }
    if (!ws) return ASTERIA_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return ASTERIA_INVALID_ARG;   // workspace must be 256-byte aligned
    // the first factor must fit: checked before anything touches the device
    if (refresh_fixed_bytes(n_all) + refresh_factor_bytes(f[0].n) > ws_bytes) return ASTERIA_WORKSPACE_TOO_SMALL;
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_);
    constexpr size_t chol_lds = CHOL_LDS_BYTES;
    static bool chol_configured[MAX_DEVICES] = {};
    ASTERIA_HIP_TRY(ensure_dynamic_lds(reinterpret_cast<const void *>(panel_chol_inverse_kernel), chol_lds, chol_configured));

    // the caller's permutation array holds the factors' orders one after the other
    std::vector<size_t> perm_offset(nfactors, 0);
    for (int i = 1; i < nfactors; ++i) perm_offset[i] = perm_offset[i - 1] + (size_t)f[i - 1].n;

    int first = 0;
    while (first < nfactors) {
        // largest pass that fits the workspace
        size_t used = refresh_fixed_bytes(n_all);
        int cnt = 0;
        while (first + cnt < nfactors) {
            const size_t b = refresh_factor_bytes(f[first + cnt].n);
            if (used + b > ws_bytes) break;
            used += b;
            ++cnt;
        }
        if (cnt == 0) return ASTERIA_WORKSPACE_TOO_SMALL;
        // The factors of a pass are dealt to two groups, each enqueued as a whole on a stream of its
        // own: the panel steps of a group are a chain of small launches (projection, Gram matrix,
        // a latency-bound Cholesky kernel on one workgroup per factor, application), and two chains
        // running side by side fill the gaps each leaves on the device.
        Carver cv(ws);
        auto enqueue_group = [&](std::vector<int> idx, hipStream_t stream) -> asteria_status {
        const int cnt = (int)idx.size();
        if (cnt == 0) return ASTERIA_OK;
        // largest first: the factors that have panel j are then the first count[j] of the group
        std::stable_sort(idx.begin(), idx.end(), [&](int a, int b) { return f[a].n > f[b].n; });
        const int n_max = f[idx[0]].n;
        const int np_max = (n_max + QR_PANEL - 1) / QR_PANEL;

        QrFactor *d_q = cv.take<QrFactor>(cnt);
        std::vector<QrFactor> q;
        bool any_qt = false;                       // some factor's Q^T is kept by the caller
        // off | pt | pz: see RefreshTables
        std::vector<int> ints((size_t)(np_max + 1) + 2 * (size_t)(cnt + 1), 0);
        int *off = ints.data(), *pt = off + np_max + 1, *pz = pt + cnt + 1;
        std::vector<int> count(np_max, 0);
        for (int i = 0; i < cnt; ++i) {
            const asteria_factor &a = f[idx[i]];
            const int n = a.n, ldz = ld4(n);
            QrFactor F;
            memset(&F, 0, sizeof(F));
            F.Zt = cv.take<float>((size_t)n * ldz);
            F.cbuf = cv.take<float>((size_t)QR_PANEL * ldz);
            F.gram = cv.take<double>((size_t)QR_PANEL * QR_PANEL);
            F.winv = cv.take<float>((size_t)QR_PANEL * QR_PANEL);
            F.Qout = a.X; F.n = n; F.ldz = ldz; F.ldq = a.ldx; F.bad = 0; F.run = 0; F.skip3 = 1;
            F.out_index = idx[i];
            F.Qt = a.X; F.ldqt = a.ldx;
            if (o.Xt && o.Xt[idx[i]]) { F.Qt = o.Xt[idx[i]]; F.ldqt = o.ldxt[idx[i]]; any_qt = true; }
            F.a_scale = 1.0f; F.p_scale = 1.0f; F.A = a.A; F.lda = a.lda;
            F.est = cv.take<double>((size_t)n);
            F.perm = cv.take<int>((size_t)n);
            F.perm_out = perm ? perm + perm_offset[idx[i]] : nullptr;
            q.push_back(F);
            const int tn = (n + BN - 1) / BN;
            pt[i + 1] = pt[i] + tn;
            pz[i + 1] = pz[i] + tn * tn;
            for (int j = 0; j < (n + QR_PANEL - 1) / QR_PANEL; ++j) ++count[j];
        }
        for (int j = 0; j < np_max; ++j) off[j + 1] = off[j] + count[j];
        const int tiles = pz[cnt], entries = off[np_max];
        RefreshTables rt;
        rt.z = cv.take<GemmProblem>(cnt);
        rt.t1 = cv.take<GemmProblem>(entries); rt.t2 = cv.take<GemmProblem>(entries);
        rt.t3 = cv.take<GemmProblem>(entries); rt.t4 = cv.take<GemmProblem>(entries);
        int *d_ints = cv.take<int>(ints.size());
        rt.off = d_ints; rt.pt = d_ints + np_max + 1; rt.pz = rt.pt + cnt + 1;
        GemmProblem *d_g = rt.z;
        ASTERIA_HIP_TRY(upload_async(d_q, q.data(), q.size() * sizeof(QrFactor), stream));
        ASTERIA_HIP_TRY(upload_async(d_ints, ints.data(), ints.size() * sizeof(int), stream));
        hipLaunchKernelGGL(refresh_tables_kernel, dim3((cnt + 127) / 128, np_max), dim3(128), 0, stream, d_q, cnt, rt);
        ASTERIA_HIP_TRY(hipGetLastError());
        // panel j: count[j] entries per table; tile counts of its four launches
        auto T1 = [&](int j) { return rt.t1 + off[j]; };
        auto T2 = [&](int j) { return rt.t2 + off[j]; };
        auto T3 = [&](int j) { return rt.t3 + off[j]; };
        auto T4 = [&](int j) { return rt.t4 + off[j]; };
        auto tiles1 = [&](int j) { return count[j] * j; };
        auto tiles24 = [&](int j) { return pt[count[j]]; };
        hipLaunchKernelGGL(qr_scale_kernel, dim3(cnt), dim3(64), 0, stream, d_q, cnt);
        if (o.from_identity)
            hipLaunchKernelGGL(set_identity_kernel, dim3((unsigned)std::min<size_t>(((size_t)n_max * n_max + 255) / 256, 4096), (unsigned)cnt),
                               dim3(256), 0, stream, d_q);
        const unsigned tpr32 = (unsigned)((n_max + 31) / 32);
        // a kept Q^T that the caller has not filled (or a start from the identity, which the kernel above
        // wrote to both buffers) is made from Q once; every round then leaves the new one there
        if (any_qt && !o.xt_in && !o.from_identity)
            hipLaunchKernelGGL(keep_qt_kernel, dim3(tpr32 * tpr32, (unsigned)cnt), dim3(256), 0, stream, d_q, 0);
        for (int round = 0; round < o.rounds; ++round) {
        hipLaunchKernelGGL(transpose_inplace_kernel, dim3(tpr32 * tpr32, (unsigned)cnt), dim3(256), 0, stream, d_q);
        ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2, true>(d_g, cnt, tiles, nullptr, stream)));
        if (o.sort) {
            // order the columns by q_i^T A q_i = (row i of Q^T) . (row i of Z^T), largest first: the rows of
            // Z^T are gathered in that order (A (Q P) = (A Q) P: sorting the basis first, as SOAP does, and
            // then multiplying gives the same Z)
            hipLaunchKernelGGL(sort_estimate_kernel, dim3((unsigned)((n_max + 3) / 4), (unsigned)cnt), dim3(256), 0, stream, d_q);
            hipLaunchKernelGGL(sort_rank_kernel, dim3((unsigned)((n_max + 255) / 256), (unsigned)cnt), dim3(256), 0, stream, d_q);
            hipLaunchKernelGGL(sort_gather_kernel, dim3((unsigned)n_max, (unsigned)cnt), dim3(256), 0, stream, d_q, 0);
            hipLaunchKernelGGL(sort_gather_kernel, dim3((unsigned)n_max, (unsigned)cnt), dim3(256), 0, stream, d_q, 1);
            ASTERIA_HIP_TRY(hipGetLastError());
        }
        for (int j = 0; j < np_max; ++j) {
            // sweeps of (project against the finished rows, orthonormalise the panel): the second
            // projection acts on normalised rows, so what the first normalisation amplified - the
            // residue of the first projection, O(1) for a row that was numerically dependent - is
            // removed again and a rank-deficient A Q still yields an orthogonal Q; factors in which
            // the second sweep met such a row run a third one
            const int *st_run = reinterpret_cast<const int *>(d_q) + offsetof(QrFactor, run) / sizeof(int);
            const int *st_third = reinterpret_cast<const int *>(d_q) + offsetof(QrFactor, skip3) / sizeof(int);
            for (int sweep = 0; sweep < 3; ++sweep) {
                const int *st = sweep < 2 ? st_run : st_third;
                if (j > 0) {
                    // projection coefficients: fp32 operands as two fp16 terms each (2^-22) in the second
                    // sweep and in the third, which only the factors that need it run (their rows are still
                    // normalised there: the Cholesky kernel keeps the unit scale until a panel's last sweep)
                    // first sweep: the coefficients as one fp16 term per operand, and one term of them in
                    // the update (the finished rows keep both terms, so the panel stays in the span of
                    // its own rows and the finished ones to 2^-22): what this leaves along the finished
                    // rows, 2^-11 of the coefficients, is what the second sweep removes at full accuracy
                    if (sweep == 0) {
                        ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 1, 1, true>(T1(j), count[j], tiles1(j), st, stream)));
                        ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 1, 2, true>(T2(j), count[j], tiles24(j), st, stream)));
                    } else if (sweep == 1) {
                        ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2, true>(T1(j), count[j], tiles1(j), st, stream)));
                        ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2, true>(T2(j), count[j], tiles24(j), st, stream)));
                    } else {
                        ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2, true>(T1(j), count[j], tiles1(j), st, stream)));
                        ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2, true>(T2(j), count[j], tiles24(j), st, stream)));
                    }
                }
                ASTERIA_HIP_TRY((launch_gemm_grouped<double, float, float, false, false>(T3(j), count[j], count[j], st, stream)));
                hipLaunchKernelGGL(panel_chol_inverse_kernel, dim3((unsigned)count[j]), dim3(CHOL_THREADS), chol_lds, stream, d_q, j, sweep);
                ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, true>(T4(j), count[j], tiles24(j), st, stream)));
            }
            // the finished panel goes to the caller's Q as columns
            hipLaunchKernelGGL(transpose_panel_kernel, dim3((QR_PANEL / 32) * ((n_max + 31) / 32), (unsigned)count[j]),
                               dim3(256), 0, stream, d_q, j);
        }
        if (any_qt)
            hipLaunchKernelGGL(keep_qt_kernel, dim3(tpr32 * tpr32, (unsigned)cnt), dim3(256), 0, stream, d_q, 1);
        }   // rounds
        hipLaunchKernelGGL(qr_info_kernel, dim3((cnt + 127) / 128), dim3(128), 0, stream, d_q, cnt, info);
        ASTERIA_HIP_TRY(hipGetLastError());
        return ASTERIA_OK;
        };
        if (n_aux < 2 || cnt < n_aux) {
            std::vector<int> all(cnt);
            for (int i = 0; i < cnt; ++i) all[i] = first + i;
            hipStream_t s0 = (n_aux == 1) ? reinterpret_cast<hipStream_t>(aux_streams[0]) : stream;
            hipEvent_t fork = nullptr, join = nullptr;
            if (n_aux == 1) {
                ASTERIA_HIP_TRY(hipEventCreateWithFlags(&fork, hipEventDisableTiming));
                ASTERIA_HIP_TRY(hipEventCreateWithFlags(&join, hipEventDisableTiming));
                ASTERIA_HIP_TRY(hipEventRecord(fork, stream));
                ASTERIA_HIP_TRY(hipStreamWaitEvent(s0, fork, 0));
            }
            const asteria_status st = enqueue_group(all, s0);
            if (n_aux == 1) {
                if (st == ASTERIA_OK) {
                    ASTERIA_HIP_TRY(hipEventRecord(join, s0));
                    ASTERIA_HIP_TRY(hipStreamWaitEvent(stream, join, 0));
                }
                (void)hipEventDestroy(fork);        // released once the recorded work has passed them
                (void)hipEventDestroy(join);
            }
            if (st != ASTERIA_OK) return st;
        } else {
            // fork: every auxiliary stream starts after everything already enqueued on the caller's
            // stream (the previous pass included); join: the caller's stream continues after all of
            // them.  The events live for this call only (destroying a recorded event releases it once
            // the work it marks has completed).
            std::vector<std::vector<int>> grp(n_aux);
            for (int i = 0; i < cnt; ++i) grp[i % n_aux].push_back(first + i);
            hipEvent_t fork = nullptr;
            ASTERIA_HIP_TRY(hipEventCreateWithFlags(&fork, hipEventDisableTiming));
            ASTERIA_HIP_TRY(hipEventRecord(fork, stream));
            asteria_status st = ASTERIA_OK;
            for (int g2 = 0; g2 < n_aux && st == ASTERIA_OK; ++g2) {
                hipStream_t sg = reinterpret_cast<hipStream_t>(aux_streams[g2]);
                hipEvent_t join = nullptr;
                if (hipEventCreateWithFlags(&join, hipEventDisableTiming) != hipSuccess ||
                    hipStreamWaitEvent(sg, fork, 0) != hipSuccess) {
                    if (join) (void)hipEventDestroy(join);
                    st = ASTERIA_HIP_ERROR;
                    break;
                }
                st = enqueue_group(grp[g2], sg);
                if (st == ASTERIA_OK && (hipEventRecord(join, sg) != hipSuccess ||
                                         hipStreamWaitEvent(stream, join, 0) != hipSuccess)) st = ASTERIA_HIP_ERROR;
                (void)hipEventDestroy(join);
            }
            (void)hipEventDestroy(fork);
            if (st != ASTERIA_OK) return st;
        }

        first += cnt;
    }
    return ASTERIA_OK;
}

// ---------------------------------------------------------------------------------------------
// asteria_soap_reproject: the first moment M of asteria_soap_step lives in the rotated space of the
// bases it was accumulated in.  When a refresh replaces (Q_L, Q_R), the matrix M stands for in the
// original space, W = Q_L,old M Q_R,old^T, is re-expressed in the new bases: M <- Q_L,new^T W Q_R,new.
// Four grouped products on the bf16 matrix cores with two-term split operands, as in
// asteria_soap_step.  The second moment V is not a linear quantity; it follows the column order only
// (V[i][j] <- V[permL[i]][permR[j]], the orders a sorted refresh reports).
namespace {

struct PermuteJob {
    float *V;          // m x n, ldv
    float *tmp;        // m x n, ldw
    const int *pl, *pr;   // row / column order, or null for the identity
    int m, n, ldv, ldw;
    int row_start;
    int pad_;
};

__global__ __launch_bounds__(256) void permute_moment_kernel(const PermuteJob *jobs, int njobs, int phase)
{
    int lo = 0, hi = njobs - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (jobs[mid].row_start <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
    }
    const PermuteJob &J = jobs[lo];
    const int i = (int)blockIdx.x - J.row_start;
    if (phase == 0) {
        const float *src = J.V + (size_t)(J.pl ? J.pl[i] : i) * J.ldv;
        float *dst = J.tmp + (size_t)i * J.ldw;
        for (int j = threadIdx.x; j < J.n; j += 256) dst[j] = src[J.pr ? J.pr[j] : j];
    } else {
        const float *src = J.tmp + (size_t)i * J.ldw;
        float *dst = J.V + (size_t)i * J.ldv;
        for (int j = threadIdx.x; j < J.n; j += 256) dst[j] = src[j];
    }
}

asteria_status validate_reproject(const asteria_rblock *b, int nblocks)
{
    if (!b || nblocks <= 0) return ASTERIA_INVALID_ARG;
    for (int i = 0; i < nblocks; ++i) {
        const asteria_rblock &k = b[i];
        if (k.m <= 0 || k.n <= 0) return ASTERIA_INVALID_ARG;
        if (!k.M && !k.V) return ASTERIA_INVALID_ARG;
        if (k.M && (!k.QL_old || !k.QL_new || !k.QR_old || !k.QR_new)) return ASTERIA_INVALID_ARG;
        if (k.M && (k.ldql_old < k.m || k.ldql_new < k.m || k.ldqr_old < k.n || k.ldqr_new < k.n || k.ldm < k.n))
            return ASTERIA_INVALID_ARG;
        if (k.V && k.ldv < k.n) return ASTERIA_INVALID_ARG;
    }
    return ASTERIA_OK;
}

}  // namespace

extern "C" size_t asteria_soap_reproject_workspace_bytes(const asteria_rblock *blocks, int nblocks)
{
    if (!blocks || nblocks <= 0) return 0;
    size_t bytes = 4 * Carver::need((size_t)nblocks, sizeof(GemmProblem)) + Carver::need((size_t)nblocks, sizeof(PermuteJob)) +
                   Carver::need(2 * (size_t)nblocks, sizeof(TransposeF32Job)) + 2048;
    for (int i = 0; i < nblocks; ++i) {
        const int m = blocks[i].m, n = blocks[i].n;
        bytes += Carver::need((size_t)m * ld4(n), sizeof(float));          // W, also the copy of V while it is permuted
        bytes += Carver::need((size_t)n * ld4(m), sizeof(float));          // transposed intermediate (n x m)
        bytes += Carver::need((size_t)m * ld4(m), sizeof(float));          // Q_L,new^T
        bytes += Carver::need((size_t)n * ld4(n), sizeof(float));          // Q_R,new^T
    }
    return bytes;
}

extern "C" asteria_status asteria_soap_reproject(const asteria_rblock *blocks, int nblocks,
                                                 void *ws, size_t ws_bytes, void *stream_)
{
    asteria_status st = validate_reproject(blocks, nblocks);
    if (st != ASTERIA_OK) return st;
    if (!ws || ws_bytes < asteria_soap_reproject_workspace_bytes(blocks, nblocks)) return ASTERIA_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return ASTERIA_INVALID_ARG;
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_);

    Carver cv(ws);
    GemmProblem *d_g[4];
    for (int i = 0; i < 4; ++i) d_g[i] = cv.take<GemmProblem>(nblocks);
    PermuteJob *d_pj = cv.take<PermuteJob>(nblocks);
    TransposeF32Job *d_tj = cv.take<TransposeF32Job>(2 * (size_t)nblocks);
    std::vector<GemmProblem> g[4];
    std::vector<PermuteJob> pj;
    std::vector<TransposeF32Job> tj;
    int tiles = 0, ttiles = 0, prow = 0;
    for (int i = 0; i < nblocks; ++i) {
        const asteria_rblock &k = blocks[i];
        const int ldw = ld4(k.n), ldt = ld4(k.m), ldqlt = ld4(k.m), ldqrt = ld4(k.n);
        float *Wb = cv.take<float>((size_t)k.m * ldw);
        float *Tt = cv.take<float>((size_t)k.n * ldt);
        float *QLt = cv.take<float>((size_t)k.m * ldqlt);
        float *QRt = cv.take<float>((size_t)k.n * ldqrt);
        if (k.V && (k.permL || k.permR)) {
            PermuteJob j;
            memset(&j, 0, sizeof(j));
            j.V = k.V; j.tmp = Wb; j.pl = k.permL; j.pr = k.permR; j.m = k.m; j.n = k.n; j.ldv = k.ldv; j.ldw = ldw;
            j.row_start = prow; prow += k.m;
            pj.push_back(j);
        }
        if (!k.M) continue;
        TransposeF32Job t;
        memset(&t, 0, sizeof(t));
        t.src = k.QL_new; t.dst = QLt; t.rows = k.m; t.cols = k.m; t.lds_ = k.ldql_new; t.ldd = ldqlt;
        t.tile_start = ttiles; ttiles += ((k.m + 31) / 32) * ((k.m + 31) / 32);
        tj.push_back(t);
        t.src = k.QR_new; t.dst = QRt; t.rows = k.n; t.cols = k.n; t.lds_ = k.ldqr_new; t.ldd = ldqrt;
        t.tile_start = ttiles; ttiles += ((k.n + 31) / 32) * ((k.n + 31) / 32);
        tj.push_back(t);
        const int tm = (k.m + BM - 1) / BM, tn = (k.n + BN - 1) / BN;
        GemmProblem p;
        memset(&p, 0, sizeof(p));
        p.state_idx = -1; p.state_mask = ~0; p.alpha = 1.0f; p.beta = 0.0f;
        p.M = k.m; p.N = k.n; p.tiles_n = tn; p.tile_start = tiles;
        // a: (M Q_R,old^T)^T:  A' = M, B'(j, k) = Q_R,old[j][k]; stored transposed
        p.K = k.n; p.A = k.M; p.lda = k.ldm; p.B = k.QR_old; p.ldb = k.ldqr_old; p.C = Tt; p.ldc = ldt; p.flags = GEMM_STORE_T;
        g[0].push_back(p);
        // b: W = Q_L,old (M Q_R,old^T):  A' = Q_L,old, B' = the transposed intermediate
        p.K = k.m; p.A = k.QL_old; p.lda = k.ldql_old; p.B = Tt; p.ldb = ldt; p.C = Wb; p.ldc = ldw; p.flags = 0;
        g[1].push_back(p);
        // c: (W Q_R,new)^T:  A' = W, B'(j, k) = Q_R,new[k][j] = its transposed copy; stored transposed
        p.K = k.n; p.A = Wb; p.lda = ldw; p.B = QRt; p.ldb = ldqrt; p.C = Tt; p.ldc = ldt; p.flags = GEMM_STORE_T;
        g[2].push_back(p);
        // d: M = Q_L,new^T (W Q_R,new):  A' = Q_L,new^T, B' = the transposed intermediate
        p.K = k.m; p.A = QLt; p.lda = ldqlt; p.B = Tt; p.ldb = ldt; p.C = k.M; p.ldc = k.ldm; p.flags = 0;
        g[3].push_back(p);
        tiles += tm * tn;
    }
    // V first: its copy uses the W buffer of the block
    if (!pj.empty()) {
        ASTERIA_HIP_TRY(upload_async(d_pj, pj.data(), pj.size() * sizeof(PermuteJob), stream));
        for (int phase = 0; phase < 2; ++phase)
            hipLaunchKernelGGL(permute_moment_kernel, dim3(prow), dim3(256), 0, stream, d_pj, (int)pj.size(), phase);
        ASTERIA_HIP_TRY(hipGetLastError());
    }
    if (g[0].empty()) return ASTERIA_OK;
    ASTERIA_HIP_TRY(upload_async(d_tj, tj.data(), tj.size() * sizeof(TransposeF32Job), stream));
    hipLaunchKernelGGL(transpose_f32_kernel, dim3(ttiles), dim3(256), 0, stream, d_tj, (int)tj.size());
    ASTERIA_HIP_TRY(hipGetLastError());
    for (int i = 0; i < 4; ++i) {
        ASTERIA_HIP_TRY(upload_async(d_g[i], g[i].data(), g[i].size() * sizeof(GemmProblem), stream));
        ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2>(d_g[i], (int)g[i].size(), tiles, nullptr, stream)));
    }
    return ASTERIA_OK;
}
