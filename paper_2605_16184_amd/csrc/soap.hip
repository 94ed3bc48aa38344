// SOAP variant (paper Eq. 2):  N = Q_L phi(Q_L^T G Q_R) Q_R^T with phi = Adam in the rotated
// basis (asteria_soap_step), and the eigenbasis refresh Q <- qr(A Q).Q (asteria_soap_refresh).
//
// soap_step:   four grouped fp32-MFMA GEMMs (rotate in: G Q_R, then Q_L^T (.); rotate out:
//              N' Q_R^T, then Q_L (.)) around one HBM-streaming Adam kernel.  Q_L / Q_R stay
//              fp32 operands: a bf16 cast of an eigenbasis costs 0.1-0.5 relative error in N.
// soap_refresh: Z^T = Q^T A by one grouped GEMM (columns of Z become contiguous rows), then a
//              Householder QR that walks those rows with one workgroup per factor
//              (wavefront-reduced norms and dot products), accumulation of Q^T by applying the
//              reflectors backwards to the identity, and a transposing write-back with the
//              column signs that make diag(R) >= 0.
#include <vector>

#include "common.h"
#include "gemm.h"

using namespace asteria;

namespace {

inline int ld4(int n) { return (n + 3) & ~3; }

__device__ __forceinline__ float wave_sum_f(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

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
// Householder QR on Z^T (row c of Zt = column c of Z), one workgroup of 1024 threads per factor.
struct QrFactor {
    float *Zt;      // n x ldz, overwritten: row j keeps the reflector v_j in columns j..n-1
    float *Qt;      // n x ldz, receives Q^T
    float *Qout;    // caller's Q (n x ldq)
    float *vtv;     // n
    float *rsign;   // n: +1 / -1 multiplier of column j of Q so that diag(R) >= 0
    int n, ldz, ldq;
    int tile_start; // for the transposing write-back (square 32 x 32 tiles)
};

constexpr int QR_THREADS = 1024;
constexpr int QR_WAVES = QR_THREADS / 64;

__device__ __forceinline__ float block_sum_1024(float v, float *red)
{
    v = wave_sum_f(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.0f;
#pragma unroll
    for (int w = 0; w < QR_WAVES; ++w) t += red[w];
    return t;
}

__global__ __launch_bounds__(QR_THREADS) void householder_rows_kernel(const QrFactor *fs, int32_t *info, int first)
{
    const QrFactor &F = fs[blockIdx.x];
    const int n = F.n, ld = F.ldz;
    __shared__ float red[QR_WAVES];
    __shared__ float sh_f;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bool bad = false;

    // forward sweep: R = H_{n-1} ... H_0 Z
    for (int j = 0; j < n; ++j) {
        float *vj = F.Zt + (size_t)j * ld;
        float s = 0.0f;
        for (int i = j + threadIdx.x; i < n; i += QR_THREADS) { const float x = vj[i]; s += x * x; }
        const float nrm2 = block_sum_1024(s, red);
        if (threadIdx.x == 0) {
            const float x0 = vj[j];
            const float nrm = sqrtf(nrm2);
            const float sgn = (x0 >= 0.0f) ? 1.0f : -1.0f;
            const float v0 = x0 + sgn * nrm;
            vj[j] = v0;
            const float vt = nrm2 - x0 * x0 + v0 * v0;
            F.vtv[j] = vt;
            // R_jj = -sgn * nrm; flip column j of Q when that is negative
            F.rsign[j] = (nrm > 0.0f && sgn > 0.0f) ? -1.0f : 1.0f;
            sh_f = vt;
        }
        __syncthreads();
        const float vt = sh_f;
        if (!(vt == vt) || vt > 3.0e38f) bad = true;
        if (vt > 0.0f && !bad) {
            // every wavefront applies H_j to its share of the remaining columns of Z
            for (int c = j + 1 + wave; c < n; c += QR_WAVES) {
                float *zc = F.Zt + (size_t)c * ld;
                float d = 0.0f;
                for (int i = j + lane; i < n; i += 64) d += vj[i] * zc[i];
                d = wave_sum_f(d);
                const float f = 2.0f * d / vt;
                for (int i = j + lane; i < n; i += 64) zc[i] -= f * vj[i];
            }
        }
        __syncthreads();
    }
    // Q^T = (H_0 ... H_{n-1})^T applied to I, built backwards: rows >= j of Qt are touched by H_j
    for (int c = wave; c < n; c += QR_WAVES) {
        float *qc = F.Qt + (size_t)c * ld;
        for (int i = lane; i < n; i += 64) qc[i] = (i == c) ? 1.0f : 0.0f;
    }
    __syncthreads();
    for (int j = n - 1; j >= 0; --j) {
        const float *vj = F.Zt + (size_t)j * ld;
        const float vt = F.vtv[j];
        if (vt > 0.0f && !bad) {
            for (int c = j + wave; c < n; c += QR_WAVES) {
                float *qc = F.Qt + (size_t)c * ld;
                float d = 0.0f;
                for (int i = j + lane; i < n; i += 64) d += vj[i] * qc[i];
                d = wave_sum_f(d);
                const float f = 2.0f * d / vt;
                for (int i = j + lane; i < n; i += 64) qc[i] -= f * vj[i];
            }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0 && info) info[first + blockIdx.x] = bad ? ASTERIA_INFO_NOT_PD : ASTERIA_INFO_OK;
}

// Q[i][c] = rsign[c] * Qt[c][i], 32 x 32 tiles through LDS
__global__ __launch_bounds__(256) void transpose_sign_kernel(const QrFactor *fs, int nf)
{
    int lo = 0, hi = nf - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (fs[mid].tile_start <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
    }
    const QrFactor &F = fs[lo];
    const int lt = (int)blockIdx.x - F.tile_start;
    const int tpr = (F.n + 31) / 32;
    const int ti = lt / tpr, tj = lt % tpr;   // tile of Qt: rows c in ti, columns i in tj
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int r = ty; r < 32; r += 8) {
        const int c = ti * 32 + r, i = tj * 32 + tx;
        tile[r][tx] = (c < F.n && i < F.n) ? F.Qt[(size_t)c * F.ldz + i] * F.rsign[c] : 0.0f;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int i = tj * 32 + r, c = ti * 32 + tx;
        if (i < F.n && c < F.n) F.Qout[(size_t)i * F.ldq + c] = tile[tx][r];
    }
}

asteria_status validate_step(const asteria_sblock *b, int nblocks, float b1, float b2, float eps, int t)
{
    if (!b || nblocks <= 0 || t < 1) return ASTERIA_INVALID_ARG;
    if (!(b1 >= 0.0f && b1 < 1.0f) || !(b2 >= 0.0f && b2 < 1.0f) || !(eps >= 0.0f)) return ASTERIA_INVALID_ARG;
    for (int i = 0; i < nblocks; ++i) {
        const asteria_sblock &k = b[i];
        if (!k.G || !k.QL || !k.QR || !k.M || !k.V || !k.N) return ASTERIA_INVALID_ARG;
        if (k.m <= 0 || k.n <= 0) return ASTERIA_INVALID_ARG;
        if (k.ldg < k.n || k.ldql < k.m || k.ldqr < k.n || k.ldm < k.n || k.ldv < k.n || k.ldn < k.n)
            return ASTERIA_INVALID_ARG;
        if (!valid_dtype(k.g_dtype)) return ASTERIA_INVALID_ARG;
    }
    return ASTERIA_OK;
}

}  // namespace

extern "C" size_t asteria_soap_step_workspace_bytes(const asteria_sblock *blocks, int nblocks)
{
    if (!blocks || nblocks <= 0) return 0;
    size_t bytes = 4 * Carver::need((size_t)nblocks, sizeof(GemmProblem)) + Carver::need((size_t)nblocks, sizeof(AdamBlock)) + 2048;
    for (int i = 0; i < nblocks; ++i)
        bytes += 2 * Carver::need((size_t)blocks[i].m * ld4(blocks[i].n), sizeof(float));
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
    std::vector<GemmProblem> g1[2], g2, g3, g4;
    std::vector<AdamBlock> ab;
    int tiles1[2] = {0, 0}, tiles = 0, rows = 0;
    for (int i = 0; i < nblocks; ++i) {
        const asteria_sblock &k = blocks[i];
        const int ldw = ld4(k.n);
        float *W = cv.take<float>((size_t)k.m * ldw);   // G Q_R, later N'
        float *Gr = cv.take<float>((size_t)k.m * ldw);  // G', later N' Q_R^T
        const int tm = (k.m + BM - 1) / BM, tn = (k.n + BN - 1) / BN;
        GemmProblem p;
        memset(&p, 0, sizeof(p));
        p.state_idx = -1; p.state_mask = ~0; p.alpha = 1.0f; p.beta = 0.0f;
        p.M = k.m; p.N = k.n; p.tiles_n = tn;
        // W = G Q_R            (B k-major)
        p.A = k.G; p.lda = k.ldg; p.B = k.QR; p.ldb = k.ldqr; p.K = k.n; p.C = W; p.ldc = ldw;
        p.tile_start = tiles1[k.g_dtype]; tiles1[k.g_dtype] += tm * tn;
        g1[k.g_dtype].push_back(p);
        p.tile_start = tiles;
        // G' = Q_L^T W         (A and B k-major)
        p.A = k.QL; p.lda = k.ldql; p.B = W; p.ldb = ldw; p.K = k.m; p.C = Gr; p.ldc = ldw;
        g2.push_back(p);
        // Y = N' Q_R^T         (both k-contiguous); N' lives in W, Y in Gr
        p.A = W; p.lda = ldw; p.B = k.QR; p.ldb = k.ldqr; p.K = k.n; p.C = Gr; p.ldc = ldw;
        g3.push_back(p);
        // N = Q_L Y            (B k-major)
        p.A = k.QL; p.lda = k.ldql; p.B = Gr; p.ldb = ldw; p.K = k.m; p.C = k.N; p.ldc = k.ldn;
        g4.push_back(p);
        tiles += tm * tn;
        AdamBlock a;
        a.Gr = Gr; a.M = k.M; a.V = k.V; a.Np = W; a.m = k.m; a.n = k.n; a.ldw = ldw; a.ldm = k.ldm; a.ldv = k.ldv;
        a.row_start = rows; rows += k.m;
        ab.push_back(a);
    }
    GemmProblem *d_g1b = d_g[0] + g1[0].size();
    if (!g1[0].empty()) ASTERIA_HIP_TRY(upload_async(d_g[0], g1[0].data(), g1[0].size() * sizeof(GemmProblem), stream));
    if (!g1[1].empty()) ASTERIA_HIP_TRY(upload_async(d_g1b, g1[1].data(), g1[1].size() * sizeof(GemmProblem), stream));
    ASTERIA_HIP_TRY(upload_async(d_g[1], g2.data(), g2.size() * sizeof(GemmProblem), stream));
    ASTERIA_HIP_TRY(upload_async(d_g[2], g3.data(), g3.size() * sizeof(GemmProblem), stream));
    ASTERIA_HIP_TRY(upload_async(d_g[3], g4.data(), g4.size() * sizeof(GemmProblem), stream));
    ASTERIA_HIP_TRY(upload_async(d_ab, ab.data(), ab.size() * sizeof(AdamBlock), stream));

    if (!g1[0].empty())
        ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, true>(d_g[0], (int)g1[0].size(), tiles1[0], nullptr, stream)));
    if (!g1[1].empty())
        ASTERIA_HIP_TRY((launch_gemm_grouped<float, bf16_t, float, false, true>(d_g1b, (int)g1[1].size(), tiles1[1], nullptr, stream)));
    ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, true, true>(d_g[1], nblocks, tiles, nullptr, stream)));
    const float c1 = 1.0f - powf(beta1, (float)step_t), c2 = 1.0f - powf(beta2, (float)step_t);
    hipLaunchKernelGGL(adam_rotated_kernel, dim3(rows), dim3(256), 0, stream, d_ab, nblocks, beta1, beta2,
                       adam_eps, 1.0f / c1, 1.0f / c2);
    ASTERIA_HIP_TRY(hipGetLastError());
    ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, false>(d_g[2], nblocks, tiles, nullptr, stream)));
    ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, true>(d_g[3], nblocks, tiles, nullptr, stream)));
    return ASTERIA_OK;
}

extern "C" size_t asteria_soap_refresh_workspace_bytes(const asteria_factor *f, int nfactors, size_t *min_bytes)
{
    if (min_bytes) *min_bytes = 0;
    if (!f || nfactors <= 0) return 0;
    size_t total = 4096, biggest = 0;
    for (int i = 0; i < nfactors; ++i) {
        const int n = f[i].n;
        if (n <= 0) return 0;
        const size_t b = 2 * Carver::need((size_t)n * ld4(n), sizeof(float)) + 2 * Carver::need((size_t)n, sizeof(float)) +
                         Carver::need(1, sizeof(GemmProblem)) + Carver::need(1, sizeof(QrFactor));
        total += b;
        biggest = b > biggest ? b : biggest;
    }
    if (min_bytes) *min_bytes = biggest + 4096;
    return total;
}

extern "C" asteria_status asteria_soap_refresh(const asteria_factor *f, int nfactors, int32_t *info,
                                               void *ws, size_t ws_bytes, void *stream_)
{
    if (!f || nfactors <= 0) return ASTERIA_INVALID_ARG;
    for (int i = 0; i < nfactors; ++i)
        if (!f[i].A || !f[i].X || f[i].n <= 0 || f[i].lda < f[i].n || f[i].ldx < f[i].n) return ASTERIA_INVALID_ARG;
    if (!ws) return ASTERIA_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return ASTERIA_INVALID_ARG;   // workspace must be 256-byte aligned
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_);

    int first = 0;
    while (first < nfactors) {
        // largest pass that fits the workspace
        size_t used = 4096;
        int cnt = 0;
        while (first + cnt < nfactors) {
            const int n = f[first + cnt].n;
            const size_t b = 2 * Carver::need((size_t)n * ld4(n), sizeof(float)) + 2 * Carver::need((size_t)n, sizeof(float)) +
                             Carver::need(1, sizeof(GemmProblem)) + Carver::need(1, sizeof(QrFactor));
            if (used + b > ws_bytes) break;
            used += b;
            ++cnt;
        }
        if (cnt == 0) return ASTERIA_WORKSPACE_TOO_SMALL;
        Carver cv(ws);
        GemmProblem *d_g = cv.take<GemmProblem>(cnt);
        QrFactor *d_q = cv.take<QrFactor>(cnt);
        std::vector<GemmProblem> g;
        std::vector<QrFactor> q;
        int tiles = 0, ttiles = 0;
        for (int i = 0; i < cnt; ++i) {
            const asteria_factor &a = f[first + i];
            const int n = a.n, ldz = ld4(n);
            QrFactor F;
            F.Zt = cv.take<float>((size_t)n * ldz);
            F.Qt = cv.take<float>((size_t)n * ldz);
            F.vtv = cv.take<float>(n);
            F.rsign = cv.take<float>(n);
            F.Qout = a.X; F.n = n; F.ldz = ldz; F.ldq = a.ldx;
            F.tile_start = ttiles;
            const int tpr = (n + 31) / 32;
            ttiles += tpr * tpr;
            q.push_back(F);
            // Z^T = Q^T A : A'(i, k) = Q[k][i] (k-major), B'(j, k) = A[j][k] (k-contiguous, A symmetric)
            GemmProblem p;
            memset(&p, 0, sizeof(p));
            p.state_idx = -1; p.state_mask = ~0; p.alpha = 1.0f; p.beta = 0.0f;
            p.M = p.N = p.K = n;
            const int tn = (n + BN - 1) / BN;
            p.tiles_n = tn;
            p.A = a.X; p.lda = a.ldx; p.B = a.A; p.ldb = a.lda; p.C = F.Zt; p.ldc = ldz;
            p.tile_start = tiles; tiles += tn * tn;
            g.push_back(p);
        }
        ASTERIA_HIP_TRY(upload_async(d_g, g.data(), g.size() * sizeof(GemmProblem), stream));
        ASTERIA_HIP_TRY(upload_async(d_q, q.data(), q.size() * sizeof(QrFactor), stream));
        ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, true, false>(d_g, cnt, tiles, nullptr, stream)));
        hipLaunchKernelGGL(householder_rows_kernel, dim3(cnt), dim3(QR_THREADS), 0, stream, d_q, info, first);
        hipLaunchKernelGGL(transpose_sign_kernel, dim3(ttiles), dim3(256), 0, stream, d_q, cnt);
        ASTERIA_HIP_TRY(hipGetLastError());
        first += cnt;
    }
    return ASTERIA_OK;
}
