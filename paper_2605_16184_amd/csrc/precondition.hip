// asteria_precondition: P = X_L G X_R for a batch of blocks (paper Eq. 1).
//
// Two chained grouped GEMMs with fp32 accumulation.  A plain bf16 cast of X_L / X_R would cost
// about 1e-2 relative error in P at condition numbers near 1e6, so the roots are never rounded
// to a single bf16:
//   bf16 gradients (the training case): bf16 matrix cores with the fp32 operands split into
//     hi + lo bf16 terms on the fly (about 16 bits kept):
//       U^T = X_R G^T   (X_R split, G exact: 2 MFMA passes; both operands k-contiguous)
//       P   = X_L U     (X_L and U^T split: 3 MFMA passes; both operands k-contiguous); blocks whose
//                       shapes fill whole 256 x 256 tiles take the 8-wavefront kernel of pgemm.h
//   fp32 gradients: fp32 matrix cores,  U = G X_R  then  P = X_L U  (U read k-major).
#include <vector>

#include "common.h"
#include "gemm.h"
#include "gemm_bf16.h"
#include "pgemm.h"

using namespace asteria;

namespace {

inline int ld4(int n) { return (n + 3) & ~3; }

asteria_status validate(const asteria_pblock *b, int nblocks)
{
    if (!b || nblocks <= 0) return ASTERIA_INVALID_ARG;
    for (int i = 0; i < nblocks; ++i) {
        const asteria_pblock &k = b[i];
        if (!k.XL || !k.G || !k.XR || !k.P) return ASTERIA_INVALID_ARG;
        if (k.m <= 0 || k.n <= 0) return ASTERIA_INVALID_ARG;
        if (k.ldxl < k.m || k.ldg < k.n || k.ldxr < k.n || k.ldp < k.n) return ASTERIA_INVALID_ARG;
        if (!valid_dtype(k.g_dtype) || !valid_dtype(k.p_dtype)) return ASTERIA_INVALID_ARG;
    }
    return ASTERIA_OK;
}

size_t table_bytes(int nblocks)
{
    return 2 * Carver::need((size_t)nblocks, sizeof(GemmProblem)) + Carver::need((size_t)nblocks, sizeof(PlaneProblem)) + 512;
}

}  // namespace

extern "C" size_t asteria_precondition_workspace_bytes(const asteria_pblock *blocks, int nblocks)
{
    if (!blocks || nblocks <= 0) return 0;
    size_t bytes = table_bytes(nblocks);
    for (int i = 0; i < nblocks; ++i) {
        const asteria_pblock &k = blocks[i];
        const size_t elems = (k.g_dtype == ASTERIA_BF16) ? (size_t)k.n * ld4(k.m) : (size_t)k.m * ld4(k.n);
        bytes += Carver::need(elems, sizeof(float));
    }
    return bytes;
}

extern "C" asteria_status asteria_precondition(const asteria_pblock *blocks, int nblocks,
                                               void *ws, size_t ws_bytes, void *stream_)
{
    asteria_status st = validate(blocks, nblocks);
    if (st != ASTERIA_OK) return st;
    if (!ws || ws_bytes < asteria_precondition_workspace_bytes(blocks, nblocks)) return ASTERIA_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return ASTERIA_INVALID_ARG;   // workspace must be 256-byte aligned
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_);

    Carver cv(ws);
    GemmProblem *d1 = cv.take<GemmProblem>(nblocks);
    GemmProblem *d2 = cv.take<GemmProblem>(nblocks);
    PlaneProblem *d2f = cv.take<PlaneProblem>(nblocks);
    std::vector<PlaneProblem> p2f;       // second product of bf16 blocks that fill whole 256 x 256 tiles
    int tiles2f = 0;
    // problems are grouped by gradient dtype: one launch per stage and dtype
    std::vector<GemmProblem> p1[2], p2[2];
    int tiles1[2] = {0, 0}, tiles2[2] = {0, 0};
    for (int i = 0; i < nblocks; ++i) {
        const asteria_pblock &k = blocks[i];
        const int d = k.g_dtype;
        const int tm = (k.m + BM - 1) / BM, tn = (k.n + BN - 1) / BN;
        GemmProblem p;
        memset(&p, 0, sizeof(p));
        p.state_idx = -1; p.state_mask = ~0;
        p.alpha = 1.0f; p.beta = 0.0f;
        if (d == ASTERIA_BF16) {
            const int ldu = ld4(k.m);
            float *Ut = cv.take<float>((size_t)k.n * ldu);
            // U^T = X_R G^T : rows of X_R against rows of G, contraction over n
            p.M = k.n; p.N = k.m; p.K = k.n; p.tiles_n = tm;
            p.A = k.XR; p.lda = k.ldxr; p.B = k.G; p.ldb = k.ldg; p.C = Ut; p.ldc = ldu; p.flags = 0;
            p.tile_start = tiles1[d]; tiles1[d] += tn * tm;
            p1[d].push_back(p);
            // P = X_L U : rows of X_L against rows of U^T, contraction over m
            p.M = k.m; p.N = k.n; p.K = k.m; p.tiles_n = tn;
            if (k.p_dtype == ASTERIA_F32 && pg_f32_operand_ok(k.XL, k.m, k.m, k.ldxl) && pg_f32_operand_ok(Ut, k.n, k.m, ldu)) {
                PlaneProblem q;
                memset(&q, 0, sizeof(q));
                q.A = k.XL; q.lda = k.ldxl; q.B = Ut; q.ldb = ldu;
                q.C32 = reinterpret_cast<float *>(k.P); q.ldc32 = k.ldp;
                q.M = k.m; q.N = k.n; q.K = k.m;
                q.tiles_n = k.n / PgF32x2::TN;
                q.tile_start = tiles2f; tiles2f += (k.m / PgF32x2::TM) * q.tiles_n;
                q.state_idx = -1; q.state_mask = ~0; q.alpha = 1.0f; q.beta = 0.0f;
                p2f.push_back(q);
            } else {
                p.A = k.XL; p.lda = k.ldxl; p.B = Ut; p.ldb = ldu; p.C = k.P; p.ldc = k.ldp;
                p.flags = (k.p_dtype == ASTERIA_BF16) ? GEMM_C_BF16 : 0;
                p.tile_start = tiles2[d]; tiles2[d] += tm * tn;
                p2[d].push_back(p);
            }
        } else {
            const int ldu = ld4(k.n);
            float *U = cv.take<float>((size_t)k.m * ldu);
            p.M = k.m; p.N = k.n; p.tiles_n = tn;
            // U = G X_R
            p.A = k.G; p.lda = k.ldg; p.B = k.XR; p.ldb = k.ldxr; p.K = k.n; p.C = U; p.ldc = ldu; p.flags = 0;
            p.tile_start = tiles1[d]; tiles1[d] += tm * tn;
            p1[d].push_back(p);
            // P = X_L U
            p.A = k.XL; p.lda = k.ldxl; p.B = U; p.ldb = ldu; p.K = k.m; p.C = k.P; p.ldc = k.ldp;
            p.flags = (k.p_dtype == ASTERIA_BF16) ? GEMM_C_BF16 : 0;
            p.tile_start = tiles2[d]; tiles2[d] += tm * tn;
            p2[d].push_back(p);
        }
    }
    GemmProblem *d1b = d1 + p1[0].size(), *d2b = d2 + p2[0].size();
    if (!p1[0].empty()) ASTERIA_HIP_TRY(upload_async(d1, p1[0].data(), p1[0].size() * sizeof(GemmProblem), stream));
    if (!p1[1].empty()) ASTERIA_HIP_TRY(upload_async(d1b, p1[1].data(), p1[1].size() * sizeof(GemmProblem), stream));
    if (!p2[0].empty()) ASTERIA_HIP_TRY(upload_async(d2, p2[0].data(), p2[0].size() * sizeof(GemmProblem), stream));
    if (!p2[1].empty()) ASTERIA_HIP_TRY(upload_async(d2b, p2[1].data(), p2[1].size() * sizeof(GemmProblem), stream));
    if (!p1[0].empty()) {
        ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, false>(d1, (int)p1[0].size(), tiles1[0], nullptr, stream)));
        ASTERIA_HIP_TRY((launch_gemm_grouped<float, float, float, false, true>(d2, (int)p2[0].size(), tiles2[0], nullptr, stream)));
    }
    if (!p1[1].empty()) {
        ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, bf16_t, 2, 1>(d1b, (int)p1[1].size(), tiles1[1], nullptr, stream)));
        if (!p2[1].empty())
            ASTERIA_HIP_TRY((launch_gemm_bf16_grouped<float, float, 2, 2>(d2b, (int)p2[1].size(), tiles2[1], nullptr, stream)));
        if (!p2f.empty()) {
            ASTERIA_HIP_TRY(upload_async(d2f, p2f.data(), p2f.size() * sizeof(PlaneProblem), stream));
            ASTERIA_HIP_TRY((launch_pgemm<PgF32x2>(d2f, (int)p2f.size(), tiles2f, nullptr, stream, 513)));
        }
    }
    return ASTERIA_OK;
}
