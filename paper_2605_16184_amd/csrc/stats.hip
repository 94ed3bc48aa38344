// asteria_stats_update: L <- beta L + (1-beta) G G^T, R <- beta R + (1-beta) G^T G for a batch
// of blocks (the Kronecker-factor statistics kept on the GPU; paper Sec. I, Sec. III-B).
//
// Both products are symmetric grouped GEMMs on the matrix cores with the EMA fused in the
// epilogue; only tiles on/below the diagonal are computed and mirrored.
//   bf16 gradients: bf16 MFMA (products exact in fp32), guard-free kernel of pgemm.h (16-byte row
//     pieces, LDS-staged epilogue with vector loads of the old L / R).  G G^T reads G as is
//     (k-contiguous).  G^T G reads G as is too when G is 16-byte aligned and fills whole tiles:
//     its operands are then k-major, staged as they lie and transposed by the LDS transpose reads
//     of gfx950.  Otherwise a transposed bf16 copy of G, zero-padded to whole tiles, is written to
//     the workspace first and read k-contiguous.  A G G^T whose operand is unaligned or ragged
//     takes the guarded kernel.
//   fp32 gradients: fp32 MFMA; G^T G reads G k-major, no copy.
//   Blocks that ask for fp64 accumulation (acc = ASTERIA_ACC_F64): products and sums on the fp64
//     matrix cores from the bf16 / fp32 data (every product exact, sums to 2^-53), the EMA in fp64
//     and one rounding to the fp32 L / R; G^T G reads G k-major, no copy.
#include <vector>

#include "common.h"
#include "gemm.h"
#include "gemm_bf16.h"
#include "pgemm.h"

using namespace asteria;

namespace {

inline int pad_to(int n, int q) { return (n + q - 1) / q * q; }

// guard-free kernel for the statistics: one bf16 term per operand, 128 x 128 tiles, slabs of 64
using StatsShape = PgShape<1, 1, PG_PAIRS_1, 2, 2, 2, 2, 64, 1, 0, false, false, true>;
constexpr int ST_TILE = StatsShape::TM;   // 128
constexpr int ST_BK = StatsShape::BK;     // 64

// G^T for a batch of bf16 blocks: 64 x 64 tiles through LDS, reads and writes along rows.  The
// destination is padded to n_pad x m_pad (whole tiles of the consumer) and the padding is zero.
struct TransposeJob {
    const uint16_t *src;   // m x n, ld = lds_
    uint16_t *dst;         // n_pad x m_pad, ld = ldd
    int m, n, lds_, ldd;
    int m_pad, n_pad;
    int tile_start;
    int pad_;
};

__global__ __launch_bounds__(256) void transpose_bf16_kernel(const TransposeJob *jobs, int njobs)
{
    int lo = 0, hi = njobs - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (jobs[mid].tile_start <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
    }
    const TransposeJob &J = jobs[lo];
    const int lt = (int)blockIdx.x - J.tile_start;
    const int tcols = J.n_pad / 64;
    const int ti = lt / tcols, tj = lt % tcols;       // tile of src: rows ti, columns tj
    __shared__ uint16_t tile[64][66];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int rr = ty; rr < 64; rr += 4) {
        const int r = ti * 64 + rr, c = tj * 64 + tx;
        tile[rr][tx] = (r < J.m && c < J.n) ? J.src[(size_t)r * J.lds_ + c] : (uint16_t)0;
    }
    __syncthreads();
    for (int rr = ty; rr < 64; rr += 4) {
        const int r = tj * 64 + rr, c = ti * 64 + tx;  // element (r, c) of dst = src(c, r), zero in the padding
        J.dst[(size_t)r * J.ldd + c] = tile[tx][rr];
    }
}

struct StatsTables {
    std::vector<GemmProblem> L[2], R[2];   // by dtype (guarded kernels)
    int tilesL[2] = {0, 0}, tilesR[2] = {0, 0};
    std::vector<GemmProblem> L64[2], R64[2];   // by dtype: fp64 accumulation
    int tilesL64[2] = {0, 0}, tilesR64[2] = {0, 0};
    std::vector<PlaneProblem> fast;        // bf16 problems for the guard-free kernel (L and R sides)
    int tiles_fast = 0;
};

// G itself can feed the guard-free kernel: 16-byte aligned rows, whole tiles and slabs
inline bool fast_operand(const void *p, int rows, int k, int ld)
{
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0 && (ld % 8) == 0 && (rows % ST_TILE) == 0 && (k % ST_BK) == 0;
}

// G can feed G^T G directly (k-major operands): columns fill whole tiles, rows whole slabs
inline bool kmajor_operand(const void *p, int m, int n, int ld)
{
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0 && (ld % 8) == 0 && (n % ST_TILE) == 0 && (m % ST_BK) == 0;
}

inline PlaneProblem fast_problem(const void *G, int rows, int k, int ld, float *C, int ldc, float beta, int tile_start,
                                 bool packed = false)
{
    PlaneProblem q;
    memset(&q, 0, sizeof(q));
    q.A = reinterpret_cast<const uint16_t *>(G); q.B = q.A;
    q.lda = ld; q.ldb = ld;
    q.C32 = C; q.ldc32 = ldc;
    q.M = rows; q.N = rows; q.K = k;
    q.tile_start = tile_start;
    q.state_idx = -1; q.state_mask = ~0;
    q.alpha = 1.0f - beta; q.beta = beta;
    q.flags = GEMM_SYM | (packed ? GEMM_C_PACKED : 0);
   
    return q;
}

asteria_status validate(const asteria_block *b, int nblocks, float beta)
{
    if (!b || nblocks <= 0) return ASTERIA_INVALID_ARG;
    if (!(beta >= 0.0f && beta < 1.0f)) return ASTERIA_INVALID_ARG;
    for (int i = 0; i < nblocks; ++i) {
        const asteria_block &k = b[i];
        if (!k.G || k.m <= 0 || k.n <= 0 || k.ldg < k.n) return ASTERIA_INVALID_ARG;
        if (!valid_dtype(k.g_dtype)) return ASTERIA_INVALID_ARG;
        if (k.acc != ASTERIA_ACC_F32 && k.acc != ASTERIA_ACC_F64) return ASTERIA_INVALID_ARG;
        if (k.lr_layout != ASTERIA_LAYOUT_FULL && k.lr_layout != ASTERIA_LAYOUT_PACKED) return ASTERIA_INVALID_ARG;
        if (!k.L && !k.R) return ASTERIA_INVALID_ARG;
        const bool full = k.lr_layout == ASTERIA_LAYOUT_FULL;      // packed: no leading dimension
        if (k.L && full && k.ldl < k.m) return ASTERIA_INVALID_ARG;
        if (k.R && full && k.ldr < k.n) return ASTERIA_INVALID_ARG;
        if (!full && ((k.L && (reinterpret_cast<uintptr_t>(k.L) & 15u)) || (k.R && (reinterpret_cast<uintptr_t>(k.R) & 15u))))
            return ASTERIA_INVALID_ARG;                            // packed tiles are read and written as 16-byte vectors
    }
    return ASTERIA_OK;
}

void build(const asteria_block *b, int nblocks, float beta, StatsTables &t)
{
    for (int i = 0; i < nblocks; ++i) {
        const asteria_block &k = b[i];
        const int d = k.g_dtype;
        GemmProblem p;
        memset(&p, 0, sizeof(p));
        p.A = k.G; p.B = k.G;
        p.lda = k.ldg; p.ldb = k.ldg;
        p.state_idx = -1; p.state_mask = ~0;
        p.alpha = 1.0f - beta; p.beta = beta;
        const bool packed = k.lr_layout == ASTERIA_LAYOUT_PACKED;
        p.flags = GEMM_SYM | (packed ? GEMM_C_PACKED : 0);
        if (k.acc == ASTERIA_ACC_F64) {
            p.flags |= GEMM_C_F32;
            if (k.L) {
                p.C = k.L; p.ldc = k.ldl; p.M = k.m; p.N = k.m; p.K = k.n;
                p.tile_start = t.tilesL64[d];
                t.tilesL64[d] += tri_tiles(k.m);
                t.L64[d].push_back(p);
            }
            if (k.R) {
                p.C = k.R; p.ldc = k.ldr; p.M = k.n; p.N = k.n; p.K = k.m;
                p.tile_start = t.tilesR64[d];
                t.tilesR64[d] += tri_tiles(k.n);
                t.R64[d].push_back(p);
            }
            continue;
        }
        if (k.L) {
            if (d == ASTERIA_BF16 && fast_operand(k.G, k.m, k.n, k.ldg)) {
                t.fast.push_back(fast_problem(k.G, k.m, k.n, k.ldg, k.L, k.ldl, beta, t.tiles_fast, packed));
                t.tiles_fast += pg_tri_tiles(k.m, ST_TILE);
            } else {
                p.C = k.L; p.ldc = k.ldl; p.M = k.m; p.N = k.m; p.K = k.n;
                p.tile_start = t.tilesL[d];
                t.tilesL[d] += tri_tiles(k.m);
                t.L[d].push_back(p);
            }
        }
        if (k.R && d != ASTERIA_BF16) {      // bf16: the transposed padded copy always feeds the guard-free kernel
            p.C = k.R; p.ldc = k.ldr; p.M = k.n; p.N = k.n; p.K = k.m;
            p.tile_start = t.tilesR[d];
            t.tilesR[d] += tri_tiles(k.n);
            t.R[d].push_back(p);
        }
    }
}

}  // namespace

extern "C" size_t asteria_stats_update_workspace_bytes(const asteria_block *blocks, int nblocks)
{
    if (!blocks || nblocks <= 0) return 0;
    size_t bytes = 4 * Carver::need((size_t)nblocks, sizeof(GemmProblem)) +
                   Carver::need(2 * (size_t)nblocks, sizeof(PlaneProblem)) +
                   Carver::need((size_t)nblocks, sizeof(TransposeJob)) + 8 * 256;
    for (int i = 0; i < nblocks; ++i)
        if (blocks[i].g_dtype == ASTERIA_BF16 && blocks[i].acc != ASTERIA_ACC_F64 && blocks[i].R && blocks[i].m > 0 &&
            blocks[i].n > 0 && !kmajor_operand(blocks[i].G, blocks[i].m, blocks[i].n, blocks[i].ldg))
            bytes += Carver::need((size_t)pad_to(blocks[i].n, ST_TILE) * pad_to(blocks[i].m, ST_BK), sizeof(uint16_t));
    return bytes;
}

extern "C" asteria_status asteria_stats_update(const asteria_block *blocks, int nblocks, float beta,
                                               void *ws, size_t ws_bytes, void *stream_)
{
    asteria_status st = validate(blocks, nblocks, beta);
    if (st != ASTERIA_OK) return st;
    if (!ws || ws_bytes < asteria_stats_update_workspace_bytes(blocks, nblocks)) return ASTERIA_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return ASTERIA_INVALID_ARG;   // workspace must be 256-byte aligned
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_);

    StatsTables t;
    build(blocks, nblocks, beta, t);
    Carver cv(ws);
    // transposed bf16 copies for the G^T G side
    {
        std::vector<TransposeJob> jobs;
        int tiles = 0;
        TransposeJob *d_jobs = cv.take<TransposeJob>(nblocks);
        for (int i = 0; i < nblocks; ++i) {
            const asteria_block &k = blocks[i];
            if (k.g_dtype != ASTERIA_BF16 || !k.R || k.acc == ASTERIA_ACC_F64) continue;
            if (kmajor_operand(k.G, k.m, k.n, k.ldg)) {
                PlaneProblem q = fast_problem(k.G, k.n, k.m, k.ldg, k.R, k.ldr, beta, t.tiles_fast, k.lr_layout == ASTERIA_LAYOUT_PACKED);
                q.flags |= PG_KMAJOR;
                t.fast.push_back(q);
                t.tiles_fast += pg_tri_tiles(k.n, ST_TILE);
                continue;
            }
            const int n_pad = pad_to(k.n, ST_TILE), m_pad = pad_to(k.m, ST_BK);
            uint16_t *Gt = cv.take<uint16_t>((size_t)n_pad * m_pad);
            TransposeJob j;
            memset(&j, 0, sizeof(j));
            j.src = reinterpret_cast<const uint16_t *>(k.G); j.dst = Gt;
            j.m = k.m; j.n = k.n; j.lds_ = k.ldg; j.ldd = m_pad;
            j.m_pad = m_pad; j.n_pad = n_pad;
            j.tile_start = tiles;
            tiles += (m_pad / 64) * (n_pad / 64);
            jobs.push_back(j);
            // the R problem of this block reads G^T with k (= m) contiguous
            t.fast.push_back(fast_problem(Gt, k.n, k.m, m_pad, k.R, k.ldr, beta, t.tiles_fast, k.lr_layout == ASTERIA_LAYOUT_PACKED));
            t.tiles_fast += pg_tri_tiles(k.n, ST_TILE);
        }
        if (!jobs.empty()) {
            ASTERIA_HIP_TRY(upload_async(d_jobs, jobs.data(), jobs.size() * sizeof(TransposeJob), stream));
            hipLaunchKernelGGL(transpose_bf16_kernel, dim3(tiles), dim3(256), 0, stream, d_jobs, (int)jobs.size());
            ASTERIA_HIP_TRY(hipGetLastError());
        }
    }
    if (!t.fast.empty()) {
        PlaneProblem *dF = cv.take<PlaneProblem>(t.fast.size());
        ASTERIA_HIP_TRY(upload_async(dF, t.fast.data(), t.fast.size() * sizeof(PlaneProblem), stream));
        ASTERIA_HIP_TRY((launch_pgemm<StatsShape>(dF, (int)t.fast.size(), t.tiles_fast, nullptr, stream, 512)));
    }
    for (int d = 0; d < 2; ++d) {
        GemmProblem *dL = nullptr, *dR = nullptr;
        if (!t.L[d].empty()) {
            dL = cv.take<GemmProblem>(t.L[d].size());
            ASTERIA_HIP_TRY(upload_async(dL, t.L[d].data(), t.L[d].size() * sizeof(GemmProblem), stream));
        }
        if (!t.R[d].empty()) {
            dR = cv.take<GemmProblem>(t.R[d].size());
            ASTERIA_HIP_TRY(upload_async(dR, t.R[d].data(), t.R[d].size() * sizeof(GemmProblem), stream));
        }
        if (d == ASTERIA_F32) {
            if (dL) ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, false>(dL, (int)t.L[d].size(), t.tilesL[d], nullptr, stream)));
            if (dR) ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, true, true>(dR, (int)t.R[d].size(), t.tilesR[d], nullptr, stream)));
        } else {
            if (dL) ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<bf16_t, bf16_t, 1, 1>(dL, (int)t.L[d].size(), t.tilesL[d], nullptr, stream)));
            if (dR) ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<bf16_t, bf16_t, 1, 1>(dR, (int)t.R[d].size(), t.tilesR[d], nullptr, stream)));
        }
    }
    // fp64 accumulation
    for (int d = 0; d < 2; ++d) {
        GemmProblem *dL = nullptr, *dR = nullptr;
        if (!t.L64[d].empty()) {
            dL = cv.take<GemmProblem>(t.L64[d].size());
            ASTERIA_HIP_TRY(upload_async(dL, t.L64[d].data(), t.L64[d].size() * sizeof(GemmProblem), stream));
        }
        if (!t.R64[d].empty()) {
            dR = cv.take<GemmProblem>(t.R64[d].size());
            ASTERIA_HIP_TRY(upload_async(dR, t.R64[d].data(), t.R64[d].size() * sizeof(GemmProblem), stream));
        }
        if (d == ASTERIA_F32) {
            if (dL) ASTERIA_HIP_TRY((launch_gemm_grouped<double, float, float, false, false>(dL, (int)t.L64[d].size(), t.tilesL64[d], nullptr, stream)));
            if (dR) ASTERIA_HIP_TRY((launch_gemm_grouped<double, float, float, true, true>(dR, (int)t.R64[d].size(), t.tilesR64[d], nullptr, stream)));
        } else {
            if (dL) ASTERIA_HIP_TRY((launch_gemm_grouped<double, bf16_t, bf16_t, false, false>(dL, (int)t.L64[d].size(), t.tilesL64[d], nullptr, stream)));
            if (dR) ASTERIA_HIP_TRY((launch_gemm_grouped<double, bf16_t, bf16_t, true, true>(dR, (int)t.R64[d].size(), t.tilesR64[d], nullptr, stream)));
        }
    }
    return ASTERIA_OK;
}
