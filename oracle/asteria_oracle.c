/*
 * Float64 CPU oracle for the Shampoo / SOAP preconditioner pipeline.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and
 * its Python binding) may include, link, import or call this file.  It shares
 * no code with the HIP kernels.  It is deliberately plain and slow: triple-loop
 * products, a cyclic-Jacobi eigendecomposition, explicit spectral functions,
 * column-by-column Householder QR, textbook Adam.  No blocking, no fusion.
 *
 * What each function follows (paper: "Asteria", Sec. II-A):
 *   oracle_stats_update   - the Kronecker-factor statistics L, R that the
 *                           method "accumulates" (Sec. I, Sec. III-B); EMA form
 *                           L <- beta L + (1-beta) G G^T, R <- beta R + (1-beta) G^T G.
 *   oracle_inverse_root   - the inverse roots of Eq. 1, regularised:
 *                           X = (A + eps I)^(-1/p), by its spectral definition.
 *   oracle_precondition   - Eq. 1:  P = L^(-1/4) G R^(-1/4) = X_L G X_R.
 *   oracle_soap_refresh   - eigenbasis refresh used with Eq. 2: one power
 *                           iteration Z = A Q followed by Householder QR,
 *                           Q <- qr(Z).Q with diag(R) >= 0.
 *   oracle_soap_step      - Eq. 2 with phi = Adam in the rotated basis.
 *   oracle_soap_sort      - the column order SOAP gives its basis before a refresh: by the
 *                           estimated eigenvalues q_i^T A q_i, largest first.
 *   oracle_soap_reproject - the moments of Eq. 2's rotated space carried from an old pair
 *                           of bases to a new one (same matrix in the original space).
 *
 * All matrices are dense row-major doubles with leading dimension = #columns.
 * Build: gcc -O2 -fopenmp -shared -fPIC (no -ffast-math: summation order is
 * the written one).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_NOT_CONVERGED 1
#define ORACLE_NOT_PD 2
#define ORACLE_BAD_ARG 3

int oracle_version(void) { return 1; }

/* ------------------------------------------------------------------ */
/* Plain products.                                                    */
/* ------------------------------------------------------------------ */

/* C (m x n) = A (m x k) * B (k x n).  i-k-j order so the inner loop is
 * contiguous; every c_ij is still the plain sum over k in increasing k. */
static void matmul_nn(int m, int n, int k, const double *A, const double *B, double *C)
{
    for (int i = 0; i < m; ++i) {
        double *c = C + (size_t)i * n;
        for (int j = 0; j < n; ++j) c[j] = 0.0;
        for (int l = 0; l < k; ++l) {
            const double a = A[(size_t)i * k + l];
            const double *b = B + (size_t)l * n;
            for (int j = 0; j < n; ++j) c[j] += a * b[j];
        }
    }
}

/* C (m x n) = A^T * B with A stored k x m, B stored k x n. */
static void matmul_tn(int m, int n, int k, const double *A, const double *B, double *C)
{
    for (int i = 0; i < m; ++i) {
        double *c = C + (size_t)i * n;
        for (int j = 0; j < n; ++j) c[j] = 0.0;
    }
    for (int l = 0; l < k; ++l) {
        const double *a = A + (size_t)l * m;
        const double *b = B + (size_t)l * n;
        for (int i = 0; i < m; ++i) {
            const double ai = a[i];
            double *c = C + (size_t)i * n;
            for (int j = 0; j < n; ++j) c[j] += ai * b[j];
        }
    }
}

/* C (m x n) = A * B^T with A stored m x k, B stored n x k. */
static void matmul_nt(int m, int n, int k, const double *A, const double *B, double *C)
{
    for (int i = 0; i < m; ++i) {
        const double *a = A + (size_t)i * k;
        for (int j = 0; j < n; ++j) {
            const double *b = B + (size_t)j * k;
            double s = 0.0;
            for (int l = 0; l < k; ++l) s += a[l] * b[l];
            C[(size_t)i * n + j] = s;
        }
    }
}

/* ------------------------------------------------------------------ */
/* Statistics: L <- beta L + (1-beta) G G^T ; R <- beta R + (1-beta) G^T G */
/* G is m x n, L is m x m, R is n x n, L and R updated in place.       */
/* ------------------------------------------------------------------ */
int oracle_stats_update(int m, int n, const double *G, double *L, double *R, double beta)
{
    if (m <= 0 || n <= 0 || !G || !L || !R) return ORACLE_BAD_ARG;
    double *GGt = (double *)malloc(sizeof(double) * (size_t)m * m);
    double *GtG = (double *)malloc(sizeof(double) * (size_t)n * n);
    if (!GGt || !GtG) { free(GGt); free(GtG); return ORACLE_BAD_ARG; }
    matmul_nt(m, m, n, G, G, GGt);
    matmul_tn(n, n, m, G, G, GtG);
    for (size_t i = 0; i < (size_t)m * m; ++i) L[i] = beta * L[i] + (1.0 - beta) * GGt[i];
    for (size_t i = 0; i < (size_t)n * n; ++i) R[i] = beta * R[i] + (1.0 - beta) * GtG[i];
    free(GGt);
    free(GtG);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* Cyclic Jacobi eigendecomposition of a symmetric matrix.            */
/*   A = V diag(lam) V^T,  V orthogonal, eigenvectors are COLUMNS of V. */
/* Row-cyclic sweeps over (p,q), p<q.  Each rotation annihilates a_pq  */
/* with the stable small-angle choice of the tangent.  Stops when the  */
/* off-diagonal Frobenius norm is <= tol * ||A||_F.                    */
/* Internally the eigenvector matrix is kept transposed (rows) so the  */
/* updates are contiguous; it is transposed back on exit.              */
/* ------------------------------------------------------------------ */
static double offdiag_fro(int n, const double *W)
{
    double s = 0.0;
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j)
            if (i != j) s += W[(size_t)i * n + j] * W[(size_t)i * n + j];
    return sqrt(s);
}

int oracle_jacobi_eigh(int n, const double *A, double *lam, double *V,
                       double tol, int max_sweeps, int *sweeps_done)
{
    if (n <= 0 || !A || !lam || !V) return ORACLE_BAD_ARG;
    double *W = (double *)malloc(sizeof(double) * (size_t)n * n);  /* working copy of A   */
    double *Vt = (double *)malloc(sizeof(double) * (size_t)n * n); /* rows = eigenvectors */
    if (!W || !Vt) { free(W); free(Vt); return ORACLE_BAD_ARG; }
    double fro = 0.0;
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
            /* work on the symmetric part */
            const double a = 0.5 * (A[(size_t)i * n + j] + A[(size_t)j * n + i]);
            W[(size_t)i * n + j] = a;
            fro += a * a;
            Vt[(size_t)i * n + j] = (i == j) ? 1.0 : 0.0;
        }
    fro = sqrt(fro);

    int status = ORACLE_NOT_CONVERGED;
    int sweep = 0;
    for (;;) {
        if (offdiag_fro(n, W) <= tol * fro) { status = ORACLE_OK; break; }
        if (sweep == max_sweeps) break;
        for (int p = 0; p < n - 1; ++p) {
            for (int q = p + 1; q < n; ++q) {
                const double apq = W[(size_t)p * n + q];
                if (apq == 0.0) continue;
                const double app = W[(size_t)p * n + p];
                const double aqq = W[(size_t)q * n + q];
                /* tangent of the rotation angle: smaller root of t^2 + 2 tau t - 1 = 0 */
                const double tau = (aqq - app) / (2.0 * apq);
                const double t = (tau >= 0.0) ? 1.0 / (tau + sqrt(1.0 + tau * tau))
                                              : 1.0 / (tau - sqrt(1.0 + tau * tau));
                const double c = 1.0 / sqrt(1.0 + t * t);
                const double s = t * c;
                /* W <- J^T W J with J = [[c, s], [-s, c]] acting on (p,q).
                 * Rows p and q first (k != p,q), then mirror into the columns. */
                double *wp = W + (size_t)p * n;
                double *wq = W + (size_t)q * n;
                for (int k = 0; k < n; ++k) {
                    const double xp = wp[k], xq = wq[k];
                    wp[k] = c * xp - s * xq;
                    wq[k] = s * xp + c * xq;
                }
                for (int k = 0; k < n; ++k) {
                    W[(size_t)k * n + p] = wp[k];
                    W[(size_t)k * n + q] = wq[k];
                }
                wp[p] = app - t * apq;
                wq[q] = aqq + t * apq;
                wp[q] = 0.0;
                wq[p] = 0.0;
                /* V <- V J, held as rows of Vt */
                double *vp = Vt + (size_t)p * n;
                double *vq = Vt + (size_t)q * n;
                for (int k = 0; k < n; ++k) {
                    const double xp = vp[k], xq = vq[k];
                    vp[k] = c * xp - s * xq;
                    vq[k] = s * xp + c * xq;
                }
            }
        }
        ++sweep;
    }
    for (int i = 0; i < n; ++i) {
        lam[i] = W[(size_t)i * n + i];
        for (int j = 0; j < n; ++j) V[(size_t)j * n + i] = Vt[(size_t)i * n + j];
    }
    if (sweeps_done) *sweeps_done = sweep;
    free(W);
    free(Vt);
    return status;
}

/* ------------------------------------------------------------------ */
/* Inverse p-th root by its spectral definition.                      */
/*   A symmetric n x n;  lambda_max = largest eigenvalue of A;        */
/*   eps = eps_value * lambda_max   (eps_relative != 0)               */
/*       = eps_value                (eps_relative == 0)               */
/*   X = V diag((lam_i + eps)^(-1/p)) V^T.                            */
/* No clamping: if some lam_i + eps <= 0 the function returns         */
/* ORACLE_NOT_PD and leaves X untouched.                              */
/* ------------------------------------------------------------------ */
int oracle_inverse_root(int n, const double *A, int p, int eps_relative, double eps_value,
                        double *X, double *lambda_max_out, double *lam_out)
{
    if (n <= 0 || p <= 0 || !A || !X) return ORACLE_BAD_ARG;
    double *lam = (double *)malloc(sizeof(double) * (size_t)n);
    double *V = (double *)malloc(sizeof(double) * (size_t)n * n);
    if (!lam || !V) { free(lam); free(V); return ORACLE_BAD_ARG; }
    int status = oracle_jacobi_eigh(n, A, lam, V, 1e-14, 60, NULL);
    if (status != ORACLE_OK) { free(lam); free(V); return status; }
    double lmax = lam[0];
    for (int i = 1; i < n; ++i) if (lam[i] > lmax) lmax = lam[i];
    if (lambda_max_out) *lambda_max_out = lmax;
    if (lam_out) memcpy(lam_out, lam, sizeof(double) * (size_t)n);
    const double eps = eps_relative ? eps_value * lmax : eps_value;
    for (int i = 0; i < n; ++i) {
        if (!(lam[i] + eps > 0.0)) { free(lam); free(V); return ORACLE_NOT_PD; }
    }
    double *f = (double *)malloc(sizeof(double) * (size_t)n);
    for (int i = 0; i < n; ++i) f[i] = pow(lam[i] + eps, -1.0 / (double)p);
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
            double s = 0.0;
            for (int k = 0; k < n; ++k) s += V[(size_t)i * n + k] * f[k] * V[(size_t)j * n + k];
            X[(size_t)i * n + j] = s;
        }
    free(f);
    free(lam);
    free(V);
    return ORACLE_OK;
}

/* Batch of independent factors, one OpenMP thread per factor (used to time
 * the oracle on all host cores; each factor is still the serial code above). */
int oracle_inverse_root_batch(int count, const int *n, const double *const *A, int p,
                              int eps_relative, const double *eps_value,
                              double *const *X, double *lambda_max_out, int *status_out)
{
    if (count <= 0 || !n || !A || !X || !eps_value) return ORACLE_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < count; ++i) {
        double lm = 0.0;
        const int st = oracle_inverse_root(n[i], A[i], p, eps_relative, eps_value[i], X[i], &lm, NULL);
        if (lambda_max_out) lambda_max_out[i] = lm;
        if (status_out) status_out[i] = st;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* Eq. 1:  P = X_L * G * X_R   (X_L m x m, G m x n, X_R n x n).        */
/* ------------------------------------------------------------------ */
int oracle_precondition(int m, int n, const double *XL, const double *G, const double *XR, double *P)
{
    if (m <= 0 || n <= 0 || !XL || !G || !XR || !P) return ORACLE_BAD_ARG;
    double *T = (double *)malloc(sizeof(double) * (size_t)m * n);
    if (!T) return ORACLE_BAD_ARG;
    matmul_nn(m, n, m, XL, G, T);
    matmul_nn(m, n, n, T, XR, P);
    free(T);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* Householder QR of Z (n x n), column by column.                     */
/* Reflector for column j:  x = Z[j:, j],  v = x + sign(x_0) ||x|| e_0, */
/* H = I - 2 v v^T / (v^T v).  R = H_{n-1} ... H_0 Z,  Q = H_0 ... H_{n-1}. */
/* Afterwards column signs are flipped so that diag(R) >= 0.          */
/* Outputs Q (n x n) and, if Rout != NULL, the upper-triangular R.     */
/* ------------------------------------------------------------------ */
int oracle_householder_qr(int n, const double *Z, double *Q, double *Rout)
{
    if (n <= 0 || !Z || !Q) return ORACLE_BAD_ARG;
    double *R = (double *)malloc(sizeof(double) * (size_t)n * n);
    double *v = (double *)malloc(sizeof(double) * (size_t)n);
    if (!R || !v) { free(R); free(v); return ORACLE_BAD_ARG; }
    memcpy(R, Z, sizeof(double) * (size_t)n * n);
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) Q[(size_t)i * n + j] = (i == j) ? 1.0 : 0.0;

    for (int j = 0; j < n; ++j) {
        double nrm2 = 0.0;
        for (int i = j; i < n; ++i) nrm2 += R[(size_t)i * n + j] * R[(size_t)i * n + j];
        const double nrm = sqrt(nrm2);
        if (nrm == 0.0) continue; /* zero column: H = I */
        const double x0 = R[(size_t)j * n + j];
        const double sgn = (x0 >= 0.0) ? 1.0 : -1.0;
        for (int i = 0; i < j; ++i) v[i] = 0.0;
        for (int i = j; i < n; ++i) v[i] = R[(size_t)i * n + j];
        v[j] = x0 + sgn * nrm;
        double vtv = 0.0;
        for (int i = j; i < n; ++i) vtv += v[i] * v[i];
        if (vtv == 0.0) continue;
        /* R <- H R  (columns j..n-1) */
        for (int c = j; c < n; ++c) {
            double dot = 0.0;
            for (int i = j; i < n; ++i) dot += v[i] * R[(size_t)i * n + c];
            const double f = 2.0 * dot / vtv;
            for (int i = j; i < n; ++i) R[(size_t)i * n + c] -= f * v[i];
        }
        /* Q <- Q H  (all rows, columns j..n-1) */
        for (int r = 0; r < n; ++r) {
            double dot = 0.0;
            for (int i = j; i < n; ++i) dot += Q[(size_t)r * n + i] * v[i];
            const double f = 2.0 * dot / vtv;
            for (int i = j; i < n; ++i) Q[(size_t)r * n + i] -= f * v[i];
        }
    }
    /* make diag(R) non-negative: Q D, D R with D = diag(sign(r_jj)) */
    for (int j = 0; j < n; ++j) {
        if (R[(size_t)j * n + j] < 0.0) {
            for (int c = 0; c < n; ++c) R[(size_t)j * n + c] = -R[(size_t)j * n + c];
            for (int r = 0; r < n; ++r) Q[(size_t)r * n + j] = -Q[(size_t)r * n + j];
        }
    }
    if (Rout) {
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) Rout[(size_t)i * n + j] = (j >= i) ? R[(size_t)i * n + j] : 0.0;
    }
    free(R);
    free(v);
    return ORACLE_OK;
}

/* SOAP eigenbasis refresh: Q <- qr(A Q).Q  (one power iteration + QR). */
int oracle_soap_refresh(int n, const double *A, double *Q, double *Rout)
{
    if (n <= 0 || !A || !Q) return ORACLE_BAD_ARG;
    double *Z = (double *)malloc(sizeof(double) * (size_t)n * n);
    double *Qn = (double *)malloc(sizeof(double) * (size_t)n * n);
    if (!Z || !Qn) { free(Z); free(Qn); return ORACLE_BAD_ARG; }
    matmul_nn(n, n, n, A, Q, Z);
    const int st = oracle_householder_qr(n, Z, Qn, Rout);
    if (st == ORACLE_OK) memcpy(Q, Qn, sizeof(double) * (size_t)n * n);
    free(Z);
    free(Qn);
    return st;
}

/* ------------------------------------------------------------------ */
/* Eq. 2 with phi = Adam in the rotated basis, step t >= 1:            */
/*   G' = Q_L^T G Q_R                                                  */
/*   M <- b1 M + (1-b1) G' ;  V <- b2 V + (1-b2) G' o G'               */
/*   N' = (M / (1-b1^t)) / (sqrt(V / (1-b2^t)) + eps)                  */
/*   N  = Q_L N' Q_R^T                                                 */
/* M, V (m x n) are updated in place; N (m x n) is the output.         */
/* ------------------------------------------------------------------ */
int oracle_soap_step(int m, int n, const double *G, const double *QL, const double *QR,
                     double *M, double *V, double beta1, double beta2, double adam_eps,
                     int t, double *N)
{
    if (m <= 0 || n <= 0 || t < 1 || !G || !QL || !QR || !M || !V || !N) return ORACLE_BAD_ARG;
    double *T = (double *)malloc(sizeof(double) * (size_t)m * n);
    double *Gr = (double *)malloc(sizeof(double) * (size_t)m * n);
    if (!T || !Gr) { free(T); free(Gr); return ORACLE_BAD_ARG; }
    matmul_tn(m, n, m, QL, G, T);   /* T  = Q_L^T G   */
    matmul_nn(m, n, n, T, QR, Gr);  /* G' = T Q_R     */
    const double c1 = 1.0 - pow(beta1, (double)t);
    const double c2 = 1.0 - pow(beta2, (double)t);
    for (size_t i = 0; i < (size_t)m * n; ++i) {
        M[i] = beta1 * M[i] + (1.0 - beta1) * Gr[i];
        V[i] = beta2 * V[i] + (1.0 - beta2) * Gr[i] * Gr[i];
        Gr[i] = (M[i] / c1) / (sqrt(V[i] / c2) + adam_eps); /* N' */
    }
    matmul_nn(m, n, m, QL, Gr, T);  /* T = Q_L N'     */
    matmul_nt(m, n, n, T, QR, N);   /* N = T Q_R^T    */
    free(T);
    free(Gr);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* Column order of an eigenbasis estimate (SOAP, used with Eq. 2):     */
/*   est_i = q_i^T A q_i  (q_i = column i of Q);  perm = indices by     */
/*   decreasing est, ties in increasing index (a stable order);        */
/*   Q <- Q[:, perm].  est_out (optional) receives est in the OLD      */
/*   column order.                                                     */
/* ------------------------------------------------------------------ */
int oracle_soap_sort(int n, const double *A, double *Q, int *perm, double *est_out)
{
    if (n <= 0 || !A || !Q || !perm) return ORACLE_BAD_ARG;
    double *est = (double *)malloc(sizeof(double) * (size_t)n);
    double *Qs = (double *)malloc(sizeof(double) * (size_t)n * n);
    if (!est || !Qs) { free(est); free(Qs); return ORACLE_BAD_ARG; }
    for (int i = 0; i < n; ++i) {
        double s = 0.0;
        for (int k = 0; k < n; ++k) {
            double aq = 0.0;                         /* (A q_i)_k */
            for (int l = 0; l < n; ++l) aq += A[(size_t)k * n + l] * Q[(size_t)l * n + i];
            s += Q[(size_t)k * n + i] * aq;
        }
        est[i] = s;
    }
    /* insertion sort of the indices: stable, largest estimate first */
    for (int i = 0; i < n; ++i) perm[i] = i;
    for (int i = 1; i < n; ++i) {
        const int p = perm[i];
        int j = i - 1;
        while (j >= 0 && est[perm[j]] < est[p]) { perm[j + 1] = perm[j]; --j; }
        perm[j + 1] = p;
    }
    for (int r = 0; r < n; ++r)
        for (int c = 0; c < n; ++c) Qs[(size_t)r * n + c] = Q[(size_t)r * n + perm[c]];
    memcpy(Q, Qs, sizeof(double) * (size_t)n * n);
    if (est_out) memcpy(est_out, est, sizeof(double) * (size_t)n);
    free(est);
    free(Qs);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* Moments of the rotated space under a change of bases (Eq. 2):      */
/* a matrix M' held in the bases (QLo, QRo) stands for                */
/*   W = QLo M' QRo^T  in the original space; in the bases (QLn, QRn) */
/* the same W is   M'' = QLn^T W QRn.   M (m x n) is updated in place. */
/* ------------------------------------------------------------------ */
int oracle_soap_reproject(int m, int n, const double *QLo, const double *QRo,
                          const double *QLn, const double *QRn, double *M)
{
    if (m <= 0 || n <= 0 || !QLo || !QRo || !QLn || !QRn || !M) return ORACLE_BAD_ARG;
    double *T = (double *)malloc(sizeof(double) * (size_t)m * n);
    double *W = (double *)malloc(sizeof(double) * (size_t)m * n);
    if (!T || !W) { free(T); free(W); return ORACLE_BAD_ARG; }
    matmul_nn(m, n, m, QLo, M, T);    /* T = QLo M'        */
    matmul_nt(m, n, n, T, QRo, W);    /* W = T QRo^T       */
    matmul_tn(m, n, m, QLn, W, T);    /* T = QLn^T W       */
    matmul_nn(m, n, n, T, QRn, M);    /* M'' = T QRn       */
    free(T);
    free(W);
    return ORACLE_OK;
}
