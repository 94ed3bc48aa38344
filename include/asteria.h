/*
 * asteria.h - C ABI of the MI355X (gfx950) Shampoo / SOAP preconditioner pipeline.
 *
 * The library implements, for a batch of independent gradient blocks G (m x n), the
 * dense-math hot path of Kronecker-factored second-order training:
 *
 *   asteria_stats_update   L <- beta L + (1-beta) G G^T,  R <- beta R + (1-beta) G^T G
 *                          (the Kronecker-factor statistics the method accumulates on the
 *                          GPU every step; paper Sec. I, Sec. III-B "factor_matrices")
 *   asteria_inverse_root   X = (A + eps I)^(-1/p), p = 4 by default, for every factor A = L
 *                          or R (the O(d^3) inverse-root update; paper Sec. I, Sec. III-B
 *                          "inv_factor_matrices", Eq. 1)
 *   asteria_precondition   P = X_L G X_R   (paper Eq. 1)
 *   asteria_soap_refresh   Q <- qr(A Q).Q  (eigenbasis refresh used with paper Eq. 2)
 *   asteria_soap_step      N = Q_L phi(Q_L^T G Q_R) Q_R^T, phi = Adam in the rotated basis
 *                          (paper Eq. 2)
 *
 * Conventions common to every entry point
 *   - All matrix pointers are DEVICE pointers owned by the caller; descriptor arrays
 *     (asteria_block[], asteria_factor[], ...) and option structs are HOST memory and are
 *     consumed before the call returns.
 *   - Matrices are dense row-major with an explicit leading dimension counted in elements.
 *     Symmetric matrices are stored full; both triangles are read as given and both are valid
 *     on return.  Inputs and outputs must not alias unless "in place" is stated.
 *   - Blocks / factors of one call may have different shapes.
 *   - `ws` is caller-owned device scratch of `ws_bytes` bytes, 256-byte aligned; the matching
 *     *_workspace_bytes query returns the size that lets the whole batch run in one pass and
 *     (where a min_bytes pointer is given) the smallest size the call accepts.  The library
 *     itself allocates no device memory and keeps no state between calls (apart from the fixed
 *     array of asteria_inverse_root_static and the measurement aid at the end of this file).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All work is
 *     enqueued on it (asteria_soap_refresh_ex: or on streams the caller passes, ordered
 *     after and before it); no entry point waits for the device.  A call may stage its descriptor
 *     tables with hipMemcpyAsync from host memory it owns until the call returns.
 *   - Entry points are not re-entrant: call them from one host thread at a time (they remember,
 *     per device, which kernels have had their launch attributes set).
 *   - The return value reports argument / launch errors only (nothing was enqueued when it
 *     is ASTERIA_INVALID_ARG, ASTERIA_UNSUPPORTED or ASTERIA_WORKSPACE_TOO_SMALL).  Numerical
 *     outcomes are per factor and device-side (`info`, `iters`, `resid`, `lambda_max`).
 */
#ifndef ASTERIA_H
#define ASTERIA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum asteria_status {
    ASTERIA_OK = 0,
    ASTERIA_INVALID_ARG = 1,
    ASTERIA_UNSUPPORTED = 2,
    ASTERIA_WORKSPACE_TOO_SMALL = 3,
    ASTERIA_HIP_ERROR = 4,
    ASTERIA_EXCEEDS_STATIC_SCRATCH = 5 /* asteria_inverse_root_static: a factor needs more than the fixed array */
} asteria_status;

typedef enum asteria_dtype {
    ASTERIA_F32 = 0,
    ASTERIA_BF16 = 1
} asteria_dtype;

/* how asteria_stats_update accumulates a block's products */
typedef enum asteria_acc {
    ASTERIA_ACC_F32 = 0, /* fp32 sums, fp32 EMA (bf16 gradients: bf16 matrix cores, products exact)   */
    ASTERIA_ACC_F64 = 1  /* fp64 sums and EMA on the fp64 matrix cores, one rounding to the fp32 L, R */
} asteria_acc;

/* storage of a symmetric fp32 matrix (statistics L, R; any matrix given to asteria_sym_pack) */
typedef enum asteria_layout {
    ASTERIA_LAYOUT_FULL = 0,   /* dense row-major n x n with a leading dimension, both triangles valid          */
    ASTERIA_LAYOUT_PACKED = 1  /* packed lower tiles (the paper's packed triangular SPD storage, Sec. III-E):
                                  the 128 x 128 tiles on and below the diagonal, tile (ti, tj), tj <= ti, at
                                  tile index ti (ti + 1) / 2 + tj, each tile dense row-major; diagonal tiles
                                  hold both of their triangles; the last tile row / column of an n that is no
                                  multiple of 128 is padded (padding never read).  asteria_packed_elems(n)
                                  floats, 16-byte aligned base, no leading dimension: 56 % of the full storage
                                  at n = 1024.  Tiles, not a packed triangle of rows, so that every row piece
                                  stays a whole number of aligned 16-byte vectors                               */
} asteria_layout;

/* per-factor numerical outcome written to the device `info` arrays */
enum {
    ASTERIA_INFO_OK = 0,
    ASTERIA_INFO_NOT_CONVERGED = 1, /* iteration budget exhausted; X holds the last iterate      */
    ASTERIA_INFO_NOT_PD = 2         /* A + eps I not positive definite or non-finite; X undefined */
};

/* One gradient block with its two statistics (asteria_stats_update). */
typedef struct asteria_block {
    const void *G; /* device, m x n, element type g_dtype, leading dimension ldg */
    float *L;      /* device, m x m fp32, leading dimension ldl, updated in place */
    float *R;      /* device, n x n fp32, leading dimension ldr, updated in place */
    int32_t m, n;
    int32_t ldg, ldl, ldr;
    int32_t g_dtype; /* asteria_dtype */
    int32_t acc;     /* asteria_acc (0 = fp32 accumulation) */
    int32_t lr_layout; /* asteria_layout of L and R (0 = full; packed: ldl, ldr unused) */
} asteria_block;

/* One symmetric factor and the matrix produced from it. */
typedef struct asteria_factor {
    const float *A; /* device, n x n fp32 symmetric statistic (read only), leading dimension lda */
    float *X;       /* device, n x n fp32: inverse root (asteria_inverse_root, written) or
                       eigenbasis Q (asteria_soap_refresh, in place), leading dimension ldx    */
    int32_t n;
    int32_t lda, ldx;
    int32_t a_layout; /* asteria_layout of A (asteria_inverse_root only; packed: lda unused).  X is always full */
} asteria_factor;

/* One block of the preconditioned update (asteria_precondition). */
typedef struct asteria_pblock {
    const float *XL; /* device, m x m fp32 symmetric, ldxl */
    const void *G;   /* device, m x n, g_dtype, ldg        */
    const float *XR; /* device, n x n fp32 symmetric, ldxr */
    void *P;         /* device, m x n, p_dtype, ldp (written) */
    int32_t m, n;
    int32_t ldxl, ldg, ldxr, ldp;
    int32_t g_dtype, p_dtype; /* asteria_dtype */
} asteria_pblock;

/* One block of the SOAP step (asteria_soap_step). */
typedef struct asteria_sblock {
    const void *G;   /* device, m x n, g_dtype, ldg                          */
    const float *QL; /* device, m x m fp32, columns = basis vectors, ldql; NULL = identity */
    const float *QR; /* device, n x n fp32, columns = basis vectors, ldqr; NULL = identity */
    float *M;        /* device, m x n fp32 first moment in the rotated basis, in place, ldm  */
    float *V;        /* device, m x n fp32 second moment in the rotated basis, in place, ldv */
    float *N;        /* device, m x n fp32 update direction (written), ldn   */
    int32_t m, n;
    int32_t ldg, ldql, ldqr, ldm, ldv, ldn;
    int32_t g_dtype;
    /* optional: Q_L^T (m x m, ldqlt) and Q_R^T (n x n, ldqrt) kept by the caller (asteria_transpose); NULL =
       the call transposes that basis into its workspace.  Unused by one-sided blocks.               */
    int32_t ldqlt, ldqrt;
    const float *QLt;
    const float *QRt;
} asteria_sblock;

typedef enum asteria_eps_mode {
    ASTERIA_EPS_RELATIVE = 0, /* eps_i = eps[i] * lambda_max(A_i), lambda_max estimated on the device */
    ASTERIA_EPS_ABSOLUTE = 1  /* eps_i = eps[i]                                                       */
} asteria_eps_mode;

/* Options of asteria_inverse_root.  Zero-initialise and call asteria_root_opts_default. */
typedef struct asteria_root_opts {
    int32_t max_iters;     /* upper bound on coupled iterations per factor (default 40)               */
    int32_t fp64_iters;    /* leading iterations run on fp64 MFMA: -1 = choose from eps (default),
                              0 = fp32 only, >= max_iters = fp64 throughout                            */
    int32_t power_iters;   /* upper bound on the steps (one product A v each) of the lambda_max estimate
                              (default 256; the Lanczos recurrence keeps at most 128)                  */
    int32_t schedule;      /* coefficients of T = a I - g M: 1 = adapted per factor and iteration to the
                              interval known to hold M's spectrum (default; about half the iterations),
                              0 = classical coupled Newton, a = (root+1)/root, g = 1/root              */
    float stop_resid;      /* a factor takes its last step once ||M - I||_F < stop_resid (default 1e-2;
                              the step after that squares the residual)                                */
    float power_tol;       /* the lambda_max estimate stops once two consecutive steps have raised it by less
                              than power_tol^2 of itself (default 1e-3, i.e. 1e-6)                     */
    float lambda_margin;   /* spectrum is scaled by 1 / ((1 + lambda_margin) lambda_max + eps)
                              (default 0.01) so an underestimated lambda_max stays inside (0, 1]      */
    int32_t lowp_from;     /* first iteration that may run on the fp16 matrix cores with the fp32 operands
                              split into two fp16 terms (22 bits kept): -1 = choose from eps (default: right
                              after the fp64 prefix, n <= 16384; never for absolute eps),
                              >= max_iters = never                                                      */
    int32_t int8_slices;   /* how the products of the fp64 iterations are computed: 0 = on the fp64 matrix
                              cores; 4 or 5 = on the int8 matrix cores, each fp64 operand held as its
                              diagonal plus that many 7-bit slices below a per-row exponent (29 / 36 bits),
                              integer accumulation exact, result assembled in fp64 - per factor and
                              product, and only where the part this drops is estimated on the device to
                              stay below a fixed fraction (2e-5, shared among the fp64 iterations) of the
                              bottom of M's spectrum; otherwise that product runs on the fp64 cores;
                              -1 = 5 (default)                                                         */
} asteria_root_opts;

void asteria_root_opts_default(asteria_root_opts *opts);

int asteria_version(void);
const char *asteria_status_string(asteria_status s);

/* ---- statistics (paper Sec. I, Sec. III-B) -------------------------------------------------
 * For every block: L <- beta L + (1-beta) G G^T and R <- beta R + (1-beta) G^T G, products
 * accumulated in fp32 (bf16 x bf16 products are exact in fp32).  L and R come back exactly
 * symmetric (one triangle is computed, the other mirrored).  Either L or R may be NULL to skip
 * that side.  0 <= beta < 1.  A block with acc = ASTERIA_ACC_F64 is accumulated in fp64 instead
 * (exact products, fp64 sums and EMA, rounded once to fp32): L and R are then the fp32 numbers
 * nearest to the exact update, whose eigenvalues lie within about 1e-9 lambda_max of the exact
 * ones - what a relative eps of 1e-8 in asteria_inverse_root needs (with fp32 sums the smallest
 * eigenvalue of a rank-deficient statistic can fall to -2e-8 lambda_max, below such an eps).  At
 * about a tenth of the speed (fp64 matrix cores).  The workspace holds the problem tables and, for a bf16 block whose
 * G is not 16-byte aligned or does not fill whole 128 x 64 tiles, a transposed copy of G.
 * Errors: NULL G, m or n <= 0, ld too small, bad dtype, beta out of range -> INVALID_ARG.   */
size_t asteria_stats_update_workspace_bytes(const asteria_block *blocks, int nblocks);
asteria_status asteria_stats_update(const asteria_block *blocks, int nblocks, float beta,
                                    void *ws, size_t ws_bytes, void *stream);

/* ---- packed triangular storage utilities (paper Sec. III-E) ---------------------------------
 * asteria_stats_update keeps L and R of a block in packed lower tiles when the block says so (it then
 * reads and writes 4 (m^2 + n^2) (1 + 1/T) bytes instead of 8 (m^2 + n^2), T = n / 128 tiles per
 * row), and asteria_inverse_root reads such statistics directly.  The roots and eigenbases stay full:
 * they are operands of the products of asteria_precondition / asteria_soap_step, whose loaders read
 * row pieces along k.  For storing them (or anything symmetric) off the hot path:
 *   asteria_sym_pack    packed <- lower tiles of full        asteria_sym_unpack  full <- packed, both triangles
 * items: host array; full: device n x n fp32, leading dimension ld; packed: device,
 * asteria_packed_elems(n) floats, 16-byte aligned.  Errors: NULL pointers, n <= 0, ld < n -> INVALID_ARG. */
typedef struct asteria_sympair {
    float *full;
    float *packed;
    int32_t n, ld;
} asteria_sympair;
size_t asteria_packed_elems(int n);
asteria_status asteria_sym_pack(const asteria_sympair *items, int nitems, void *stream);
asteria_status asteria_sym_unpack(const asteria_sympair *items, int nitems, void *stream);

/* ---- inverse p-th roots (paper Eq. 1, Sec. III-B) ------------------------------------------
 * For every factor: X = ((A + A^T)/2 + eps I)^(-1/root), root in {2, 4} (4 = Eq. 1), by a coupled
 * matrix iteration run entirely on the device.
 *
 *   step                what the device does
 *   ------------------  --------------------------------------------------------------------------
 *   lambda_max          Lanczos process on A (three-term recurrence from a fixed start vector, one product
 *                       A v per step): the largest Ritz value, stopped per factor when it has settled
 *   scaling             s = 1 / ((1 + margin) lambda_max + eps); M_0 = s (A + eps I), X_0 = s^(1/root) I;
 *                       the spectrum of M_0 is taken to lie in [eps s / 2, 1]
 *   iteration           T = a I - g M, X <- X T, M <- T^root M; (a, g) per factor and iteration from
 *                       the interval that holds M's spectrum (`schedule` = 1) or the Newton values
 *   stop (per factor)   one more X update follows once ||M - I||_F < stop_resid, or once the interval
 *                       predicted for M's spectrum is within 1 +- 1e-2 and the measured residual is
 *                       consistent with it; under the automatic precision rules already when the image
 *                       of that interval under the next update is within 1 +- 3e-3
 *
 *   iterations          matrices  products run on
 *   ------------------  --------  ----------------------------------------------------------------
 *   first fp64_iters    fp64      int8 matrix cores (diagonal + 7-bit slices, exact integer sums, fp64
 *                                 assembly) or fp64 matrix cores, per factor and product: `int8_slices`
 *   up to lowp_from     fp32      fp32 matrix cores
 *   from lowp_from on   fp32      fp16 matrix cores, every operand split into two fp16 terms (kept to
 *                                 2^-22), scaled into the fp16 range by powers of two derived from the
 *                                 bounds the call keeps on M and X
 *
 * What the interval-based choices rely on.  A is positive semi-definite up to round-off: eigenvalues
 * down to -eps / 2 are covered by the lower end eps s / 2 (statistics accumulated in fp32 can fall
 * further below zero when eps is of the order of 1e-8 lambda_max: accumulate those with
 * ASTERIA_ACC_F64).  The largest Ritz value never exceeds lambda_max and reaches it to a few 1e-7 on
 * every workload tested (leading eigenvalues 0.4 % apart included); it stalls below only if the start
 * vector has no component along the leading eigenvectors, and `lambda_margin` (1 %) is the allowance
 * for that.  If
 * either assumption fails for a factor - an eigenvalue of M_0 outside [eps s / 2, 1] - the predicted
 * interval is wrong for it: the measured residual then disagrees with the prediction, the factor
 * falls back to the residual rule and runs until ||M - I||_F < stop_resid or max_iters, where it
 * reports ASTERIA_INFO_NOT_CONVERGED; a residual that still agrees within its tolerance
 * (1.5 sqrt(n) times the predicted deviation + 2e-3) can hide one stray eigenvalue that far from 1.
 *
 *   eps        host array, eps_count entries (1 = shared by all factors, else nfactors).
 *   info       device int32[nfactors] or NULL   (ASTERIA_INFO_*)
 *   iters      device int32[nfactors] or NULL   (number of X <- X T updates performed)
 *   resid      device float[nfactors] or NULL   (last measured ||M - I||_F)
 *   lambda_max device float[nfactors] or NULL   (the estimate used)
 * Workspace: the call splits the batch into passes that fit ws_bytes; *min_bytes is the size
 * needed for the largest single factor.
 * Errors: NULL A or X, n <= 0, ld < n, unsupported root or int8_slices, eps < 0 or non-finite,
 * eps_count not in {1, nfactors} -> INVALID_ARG / UNSUPPORTED; ws too small ->
 * WORKSPACE_TOO_SMALL.                                                                       */
/* The precision schedule asteria_inverse_root would use for these arguments (host only, nothing is
 * launched): number of leading fp64 iterations of the M-chain (T^2, T^4, T^4 M), first iteration of
 * that chain on the fp16 matrix cores (>= max_iters = never; factors larger than 16384 stay on the
 * fp32 cores under the automatic rule), and whether every X <- X T product runs on the fp16 cores
 * with split operands (1) or in the precision tier of its iteration, fp32 at least (0).  X is
 * stored in fp32 in every tier.  Any of the three outputs may be NULL.                          */
asteria_status asteria_inverse_root_plan(int root, asteria_eps_mode mode, const float *eps, int eps_count,
                                         const asteria_root_opts *opts, int32_t *fp64_iters,
                                         int32_t *lowp_from, int32_t *x_update_lowp);
size_t asteria_inverse_root_workspace_bytes(const asteria_factor *f, int nfactors,
                                            const asteria_root_opts *opts, size_t *min_bytes);
asteria_status asteria_inverse_root(const asteria_factor *f, int nfactors, int root,
                                    asteria_eps_mode mode, const float *eps, int eps_count,
                                    const asteria_root_opts *opts,
                                    int32_t *info, int32_t *iters, float *resid, float *lambda_max,
                                    void *ws, size_t ws_bytes, void *stream);

/* ---- inverse p-th roots for callers that cannot allocate ------------------------------------
 * For code that runs under HIP graph capture, tight serving loops and harnesses that forbid
 * allocation: the same computation as asteria_inverse_root with the same arguments, except that
 * the workspace is a fixed array of asteria_static_scratch_bytes() = 64 MiB inside the library's
 * device image (every GPU the library runs on holds its own copy until the process ends; its
 * address is looked up at the first call on a device).  The call allocates no device memory and
 * calls no allocating routine.  The batch is worked through in passes that fit the array, so any
 * number of factors is accepted, but each factor by itself must fit: with default options n up to
 * about 1100 (50 bytes per matrix element plus tables).  A larger factor ->
 * ASTERIA_EXCEEDS_STATIC_SCRATCH, nothing enqueued.  All calls on one GPU share that GPU's array,
 * which keeps the last call's contents (every word a call reads it has written first): calls that
 * overlap on one GPU - two streams, two threads - race; order them.                            */
size_t asteria_static_scratch_bytes(void);
asteria_status asteria_inverse_root_static(const asteria_factor *f, int nfactors, int root,
                                           asteria_eps_mode mode, const float *eps, int eps_count,
                                           const asteria_root_opts *opts,
                                           int32_t *info, int32_t *iters, float *resid, float *lambda_max,
                                           void *stream);

/* ---- preconditioned update (paper Eq. 1) ---------------------------------------------------
 * For every block: P = X_L G X_R, X_L and X_R symmetric fp32; P is written as fp32 or bf16
 * (round to nearest even).  fp32 gradients: fp32 matrix cores.  bf16 gradients: bf16 matrix cores
 * with fp32 accumulation, G exact and every fp32 operand (X_L, X_R, the intermediate) split into
 * two bf16 terms, which keeps about 16 bits of it (measured 5e-6 .. 9e-6 relative error in P).
 * Workspace holds the intermediate G X_R of every block (fp32, m x n each).                 */
size_t asteria_precondition_workspace_bytes(const asteria_pblock *blocks, int nblocks);
asteria_status asteria_precondition(const asteria_pblock *blocks, int nblocks,
                                    void *ws, size_t ws_bytes, void *stream);

/* ---- SOAP eigenbasis refresh (paper Eq. 2) -------------------------------------------------
 * For every factor: Z = A Q (one power iteration), Z = Q' R the QR factorisation with
 * diag(R) >= 0 (unique for a Z of full rank: the Q' a Householder QR with that sign convention
 * returns), and Q <- Q' in place (f[i].X is Q).  Computed by block Gram-Schmidt with
 * re-orthogonalisation over panels of 128 columns.  The large products - A Q, the projection
 * coefficients of a panel against the finished columns and their subtraction - run on the fp16
 * matrix cores with every fp32 operand split into two fp16 terms (22 bits kept) after a scaling
 * by a power of two taken from tr A, with fp32 accumulation; panel Gram matrices and their
 * Cholesky factors are fp64, the application of the inverse factor uses the fp32 matrix cores; a
 * panel whose second sweep meets a row that was numerically dependent takes a third one.  The first
 * sweep of a panel works with one fp16 term of the coefficients (the second removes what that leaves).  Columns of Z beyond its numerical rank come out as
 * an orthonormal completion.  Q is used as scratch during the call (transposed in place, then
 * overwritten panel by panel); where info reports a failure its content is unspecified.
 * asteria_soap_refresh enqueues everything on `stream`.  asteria_soap_refresh_ex takes options
 * (zero-initialise and call asteria_soap_refresh_opts_default):
 *   n_aux, aux_streams  deal the factors to n_aux (1..4) groups and enqueue each group as a whole on
 *       aux_streams[g], streams of the caller (default priority, none equal to `stream`): they start
 *       after everything already enqueued on `stream`, and `stream` waits for them before the call's
 *       work counts as done on it (events created and released inside the call).  A group's panel
 *       steps are a chain of small launches around a latency-bound Cholesky kernel; two chains side
 *       by side fill each other's gaps (1B-model workload: 186 ms with two streams, 205 ms on one).
 *   sort  1: before the power iteration the columns of Q are put in the order of decreasing
 *       estimated eigenvalue q_i^T A q_i, ties by column index (the order SOAP gives its basis; the
 *       moments of asteria_soap_step then have to follow: asteria_soap_reproject).  `perm`, device
 *       int32, the factors' orders one after the other (sum of n entries; perm[r] = input column
 *       that became column r before the QR), or NULL.
 *   from_identity  1: start from Q = I, whatever Q holds (first basis of a new statistic).
 *   rounds  number of (power iteration, QR) rounds in the call, >= 1: from the identity, a few
 *       sorted rounds are orthogonal iteration towards the eigenbasis - the device-side stand-in for
 *       the eigendecomposition SOAP starts from.  `perm` needs rounds = 1.
 *   Xt, ldxt, xt_in  a caller that keeps Q^T beside Q (asteria_soap_step reads it) passes the buffers: the
 *       call leaves the transpose of the new basis there - the rows it has orthonormalised, a plain copy -
 *       and reads the product's operand Q^T from there instead of transposing Q in place; xt_in = 1 says
 *       the buffers hold the transpose of the incoming Q already (they do after a call that was given them),
 *       otherwise the call fills them first.  Xt[i] must not be f[i].X.
 *   info  device int32[nfactors] or NULL (ASTERIA_INFO_OK, or ASTERIA_INFO_NOT_PD if a column
 *         could not be normalised: an exactly zero or non-finite column, or one that three
 *         sweeps of re-orthogonalisation did not separate from the columns before it).       */
size_t asteria_soap_refresh_workspace_bytes(const asteria_factor *f, int nfactors, size_t *min_bytes);
asteria_status asteria_soap_refresh(const asteria_factor *f, int nfactors, int32_t *info,
                                    void *ws, size_t ws_bytes, void *stream);
typedef struct asteria_soap_refresh_opts {
    int32_t sort;
    int32_t from_identity;
    int32_t rounds;
    int32_t n_aux;
    void *const *aux_streams;
    float *const *Xt;       /* NULL, or nfactors pointers (each may be NULL): device n x n fp32 buffers for Q^T */
    const int32_t *ldxt;    /* their leading dimensions (with Xt)                                            */
    int32_t xt_in;          /* 1: every Xt[i] already holds the transpose of the incoming Q                  */
} asteria_soap_refresh_opts;
void asteria_soap_refresh_opts_default(asteria_soap_refresh_opts *opts);
asteria_status asteria_soap_refresh_ex(const asteria_factor *f, int nfactors, const asteria_soap_refresh_opts *opts,
                                       int32_t *info, int32_t *perm, void *ws, size_t ws_bytes, void *stream);

/* ---- SOAP step (paper Eq. 2, phi = Adam in the rotated basis) ------------------------------
 * For every block, with step_t >= 1:
 *   G' = Q_L^T G Q_R;  M <- beta1 M + (1-beta1) G';  V <- beta2 V + (1-beta2) G' o G';
 *   N' = (M / (1-beta1^t)) / (sqrt(V / (1-beta2^t)) + adam_eps);  N = Q_L N' Q_R^T.
 * The four rotations run on the bf16 matrix cores with fp32 accumulation and every fp32 operand
 * split into two bf16 terms (bf16 G exact): about 16 bits of Q_L, Q_R and of the intermediates.
 * Workspace: G', N', one intermediate and the transposes of Q_L, Q_R of every block.  The products read
 * Q_L^T and Q_R^T along rows; a basis changes only at a refresh, so a caller may keep the transposes
 * (asteria_transpose after each refresh) and pass them in the block: the call then neither needs that
 * workspace nor moves those 8 (m^2 + n^2) bytes per step.  A passed transpose must be that of the
 * passed basis; the call does not check it.
 * One-sided blocks: QL or QR (not both) may be NULL and stands for the identity - a dimension above
 * the preconditioner cap keeps no basis.  Such a block takes one product per rotation, on the fp32
 * matrix cores with the operands read in place.                                                 */
size_t asteria_soap_step_workspace_bytes(const asteria_sblock *blocks, int nblocks);
asteria_status asteria_soap_step(const asteria_sblock *blocks, int nblocks,
                                 float beta1, float beta2, float adam_eps, int step_t,
                                 void *ws, size_t ws_bytes, void *stream);

/* ---- transposed copies (utility for asteria_soap_step) -----------------------------------------
 * dst (cols x rows, ldd) = src^T for every item (src: rows x cols, lds), 32 x 32 tiles through LDS.
 * items: host array; src, dst: device, fp32, not overlapping.  Errors: NULL pointers, rows or
 * cols <= 0, lds < cols, ldd < rows -> INVALID_ARG.                                              */
typedef struct asteria_tpair {
    const float *src;
    float *dst;
    int32_t rows, cols, lds, ldd;
} asteria_tpair;
asteria_status asteria_transpose(const asteria_tpair *items, int nitems, void *stream);

/* ---- moments under a change of bases (paper Eq. 2) ---------------------------------------------
 * asteria_soap_step keeps the Adam moments in the rotated space of (Q_L, Q_R).  After a refresh has
 * replaced the bases, the first moment is carried over so that it stands for the same matrix of the
 * original space:  M <- Q_L,new^T (Q_L,old M Q_R,old^T) Q_R,new  (the caller keeps a copy of the old
 * bases: the refresh works in place).  The second moment V is not linear in the gradient and only
 * follows the column order of a sorted refresh: V[i][j] <- V[permL[i]][permR[j]] (permL, permR: the
 * slices of asteria_soap_refresh_ex's `perm` for the block's two factors, device int32, or NULL for
 * no reordering on that side).  M or V may be NULL to skip that part.  The four products of M run on
 * the bf16 matrix cores with two-term split operands (16 bits kept), as in asteria_soap_step.
 * Workspace: two intermediates and the transposes of the new bases per block.                     */
typedef struct asteria_rblock {
    const float *QL_old, *QL_new;  /* device, m x m fp32, columns = basis vectors */
    const float *QR_old, *QR_new;  /* device, n x n fp32                           */
    float *M;                      /* device, m x n fp32, in place, or NULL        */
    float *V;                      /* device, m x n fp32, in place, or NULL        */
    const int32_t *permL, *permR;  /* device, m and n entries, or NULL             */
    int32_t m, n;
    int32_t ldql_old, ldql_new, ldqr_old, ldqr_new, ldm, ldv;
} asteria_rblock;
size_t asteria_soap_reproject_workspace_bytes(const asteria_rblock *blocks, int nblocks);
asteria_status asteria_soap_reproject(const asteria_rblock *blocks, int nblocks,
                                      void *ws, size_t ws_bytes, void *stream);

/* ---- measurement aid (not part of the method) -----------------------------------------------
 * Between asteria_profile_enable and asteria_profile_collect every grouped-GEMM launch made by
 * the entry points above is bracketed by a pair of HIP events on the caller's stream (at most
 * max_launches launches are recorded; the events are created on the host, no device memory).
 * asteria_profile_collect waits for the recorded events, writes one duration in milliseconds and
 * one kernel-kind code per launch, in launch order, into the HOST arrays ms / kind (capacity
 * cap), destroys the events, switches recording off and returns the number of entries written
 * (-1 if recording was not on).  kind codes: below 32 the fp32 / fp64 kernel, bits 1 = fp64 matrix
 * cores (else fp32), 2 = A operand bf16, 4 = B operand bf16, 8 = A read k-major, 16 = B read
 * k-major; 32..255 the 16-bit kernel, 32 + (2 = A operand bf16 in memory) + (4 = B operand bf16 in
 * memory) + (64 = A split into two terms) + (128 = B split into two terms), so 224 = both operands
 * fp32 split in two terms and 96 = A split, B one term; 256..299 the guard-free kernels (512 the
 * statistics, 513 the 256 x 256 split x split products); 300 + NS the int8-slice kernel whose planes
 * hold NS slices (304, 305).  Not thread safe.                                                    */
asteria_status asteria_profile_enable(int max_launches);
int asteria_profile_collect(float *ms, int32_t *kind, int cap);
/* Algorithmic flops (n^2 (n + 1) per symmetric product) of the products of the fp64 iterations since
 * the last asteria_profile_enable, by where the device-side decision sent them: out3[0] fp64 matrix
 * cores, out3[1] int8 cores with 4 slices, out3[2] with 5.  Waits for the device.               */
asteria_status asteria_profile_i8_flops(double *out3);

#ifdef __cplusplus
}
#endif
#endif /* ASTERIA_H */
