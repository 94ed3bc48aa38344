// asteria_stats_update: L <- beta L + (1-beta) G G^T, R <- beta R + (1-beta) G^T G for a batch
// of blocks (the Kronecker-factor statistics kept on the GPU; paper Sec. I, Sec. III-B).
//
// Both products are symmetric grouped GEMMs on the matrix cores: G G^T reads G with k
// contiguous, G^T G reads the same memory k-major, so G is never transposed in HBM.  The EMA
// is fused in the epilogue; only tiles on/below the diagonal are computed and mirrored.
#include <vector>

#include "common.h"
#include "gemm.h"

using namespace asteria;

namespace {

struct StatsTables {
    std::vector<GemmProblem> L[2], R[2];   // by dtype
    int tilesL[2] = {0, 0}, tilesR[2] = {0, 0};
};

asteria_status validate(const asteria_block *b, int nblocks, float beta)
{
    if (!b || nblocks <= 0) return ASTERIA_INVALID_ARG;
    if (!(beta >= 0.0f && beta < 1.0f)) return ASTERIA_INVALID_ARG;
    for (int i = 0; i < nblocks; ++i) {
        const asteria_block &k = b[i];
        if (!k.G || k.m <= 0 || k.n <= 0 || k.ldg < k.n) return ASTERIA_INVALID_ARG;
        if (!valid_dtype(k.g_dtype)) return ASTERIA_INVALID_ARG;
        if (!k.L && !k.R) return ASTERIA_INVALID_ARG;
        if (k.L && k.ldl < k.m) return ASTERIA_INVALID_ARG;
        if (k.R && k.ldr < k.n) return ASTERIA_INVALID_ARG;
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
        p.flags = GEMM_SYM;
        if (k.L) {
            p.C = k.L; p.ldc = k.ldl; p.M = k.m; p.N = k.m; p.K = k.n;
            p.tile_start = t.tilesL[d];
            t.tilesL[d] += tri_tiles(k.m);
            t.L[d].push_back(p);
        }
        if (k.R) {
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
    (void)blocks;
    if (nblocks <= 0) return 0;
    return 2 * Carver::need((size_t)nblocks, sizeof(GemmProblem)) + 4 * 256;
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
            if (dL) ASTERIA_HIP_TRY((launch_gemm_grouped<float, bf16_t, bf16_t, false, false>(dL, (int)t.L[d].size(), t.tilesL[d], nullptr, stream)));
            if (dR) ASTERIA_HIP_TRY((launch_gemm_grouped<float, bf16_t, bf16_t, true, true>(dR, (int)t.R[d].size(), t.tilesR[d], nullptr, stream)));
        }
    }
    return ASTERIA_OK;
}
