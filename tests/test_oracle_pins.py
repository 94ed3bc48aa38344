"""Pins for the float64 oracle: every oracle function is checked against something other
than itself - closed forms, hand-computed small cases, invariants, multi-precision brute
force (mpmath, 50 digits) and library witnesses (numpy.linalg).  CPU only.

Paper passages: Sec. II-A Eq. 1 (Shampoo), Eq. 2 (SOAP); Sec. I / III-B (statistics L, R).
"""
import math

import mpmath
import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(20260516)


def relF(a, b):
    return np.linalg.norm(np.asarray(a) - np.asarray(b)) / np.linalg.norm(np.asarray(b))


def haar(n, rng):
    q, r = np.linalg.qr(rng.standard_normal((n, n)))
    return q * np.sign(np.diag(r))


# ----------------------------------------------------------------------------- Jacobi eigh

def test_jacobi_analytic_2x2():
    lam, V, _ = oracle.jacobi_eigh(np.array([[2.0, 1.0], [1.0, 2.0]]))
    order = np.argsort(lam)
    assert np.allclose(lam[order], [1.0, 3.0], atol=1e-15)
    v1, v3 = V[:, order[0]], V[:, order[1]]
    assert abs(abs(v1 @ np.array([1.0, -1.0]) / math.sqrt(2)) - 1) < 1e-15
    assert abs(abs(v3 @ np.array([1.0, 1.0]) / math.sqrt(2)) - 1) < 1e-15


def test_jacobi_known_spectrum_from_givens_product():
    # A = W diag(d) W^T where W is an explicit product of plane rotations: spectrum is d.
    n = 6
    d = np.array([5.0, 3.0, 2.0, 1.0, 0.5, 0.25])
    W = np.eye(n)
    for (p, q, th) in [(0, 1, 0.3), (1, 2, -0.7), (2, 5, 1.1), (0, 4, 0.9), (3, 4, -0.2), (1, 5, 0.45)]:
        J = np.eye(n)
        J[p, p] = J[q, q] = math.cos(th)
        J[p, q] = math.sin(th)
        J[q, p] = -math.sin(th)
        W = W @ J
    A = W @ np.diag(d) @ W.T
    lam, V, _ = oracle.jacobi_eigh(A)
    order = np.argsort(-lam)
    assert np.allclose(lam[order], d, rtol=0, atol=1e-14)
    for k in range(n):  # eigenvectors equal W's columns up to sign
        assert abs(abs(V[:, order[k]] @ W[:, k]) - 1) < 1e-13


@pytest.mark.parametrize("n", [1, 3, 17, 64, 128])
def test_jacobi_residual_orthogonality_and_lapack_witness(n):
    B = RNG.standard_normal((n, n))
    A = B @ B.T + np.diag(RNG.uniform(0, 1, n))
    lam, V, sweeps = oracle.jacobi_eigh(A)
    assert sweeps <= 15
    assert np.linalg.norm(V @ np.diag(lam) @ V.T - A) <= 1e-13 * max(np.linalg.norm(A), 1e-300) * max(1, n / 32)
    assert np.linalg.norm(V.T @ V - np.eye(n)) <= 1e-13 * max(1, n / 16)
    assert np.allclose(np.sort(lam), np.linalg.eigvalsh(A), rtol=0, atol=1e-12 * lam.max())


def test_jacobi_graded_spectrum_small_eigenvalues():
    # log-spaced spectrum over 16 decades (as the ill-conditioned workload squares 1e0..1e-8)
    n = 48
    d = 10.0 ** np.linspace(0, -16, n)
    U = haar(n, RNG)
    A = (U * d) @ U.T
    lam, V, _ = oracle.jacobi_eigh(A)
    assert np.allclose(np.sort(lam)[::-1], d, rtol=0, atol=1e-15)


# ----------------------------------------------------------------------------- statistics

def test_stats_hand_computed_integers_nonsquare():
    G = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]])          # 2 x 3
    L0 = np.array([[2.0, 0.0], [0.0, 2.0]])
    R0 = np.zeros((3, 3))
    L, R = oracle.stats_update(G, L0, R0, 0.5)
    # G G^T = [[14, 32], [32, 77]],  G^T G = [[17,22,27],[22,29,36],[27,36,45]]
    assert np.array_equal(L, 0.5 * L0 + 0.5 * np.array([[14.0, 32.0], [32.0, 77.0]]))
    assert np.array_equal(R, 0.5 * np.array([[17.0, 22, 27], [22, 29, 36], [27, 36, 45]]))


def test_stats_trace_symmetry_and_witness():
    m, n, beta = 13, 21, 0.95
    G = RNG.standard_normal((m, n))
    S = RNG.standard_normal((m, m)); L0 = S @ S.T
    S = RNG.standard_normal((n, n)); R0 = S @ S.T
    L, R = oracle.stats_update(G, L0, R0, beta)
    assert np.array_equal(L, L.T) and np.array_equal(R, R.T)
    g2 = np.sum(G * G)
    assert math.isclose(np.trace(L), beta * np.trace(L0) + (1 - beta) * g2, rel_tol=1e-13)
    assert math.isclose(np.trace(R), beta * np.trace(R0) + (1 - beta) * g2, rel_tol=1e-13)
    assert relF(L, beta * L0 + (1 - beta) * G @ G.T) < 1e-14
    assert relF(R, beta * R0 + (1 - beta) * G.T @ G) < 1e-14
    # inputs are not modified
    assert np.array_equal(S @ S.T, R0)


def test_stats_eight_ema_steps_from_identity_condition_number():
    # 128x128 block, G ~ N(0, 0.01^2), L0 = I, 8 updates with beta = 0.95:
    # L = beta^8 I + small PSD part, so diag((L+eps)^-1/4) ~ (0.95^8)^-1/4 ~ 1.10
    n = 128
    L = np.eye(n); R = np.eye(n)
    for _ in range(8):
        G = 0.01 * RNG.standard_normal((n, n))
        L, R = oracle.stats_update(G, L, R, 0.95)
    X, lmax, lam = oracle.inverse_root(L, 1e-6)
    assert lam.max() / lam.min() < 1.05
    assert np.allclose(np.diag(X), 0.95 ** -2, rtol=5e-3)
    assert np.abs(X - np.diag(np.diag(X))).max() < 5e-3


# ----------------------------------------------------------------------------- inverse root

def test_inverse_root_identity_and_diagonal_closed_forms():
    n, eps = 7, 1e-3
    X, lmax, _ = oracle.inverse_root(np.eye(n), eps)
    assert lmax == 1.0
    assert np.allclose(X, (1 + eps) ** -0.25 * np.eye(n), rtol=0, atol=1e-15)
    d = np.array([4.0, 1.0, 0.25, 16.0, 1e-4])
    X, lmax, _ = oracle.inverse_root(np.diag(d), 1e-2, relative=True)
    assert lmax == 16.0
    assert np.allclose(X, np.diag((d + 0.16) ** -0.25), rtol=0, atol=1e-14)
    X, _, _ = oracle.inverse_root(np.diag(d), 1e-2, relative=False)
    assert np.allclose(X, np.diag((d + 1e-2) ** -0.25), rtol=0, atol=1e-14)
    X, _, _ = oracle.inverse_root(np.diag(d), 0.0, relative=False, p=2)
    assert np.allclose(X, np.diag(d ** -0.5), rtol=1e-14, atol=0)


def test_inverse_root_rank_one_statistics_closed_form():
    # G = u v^T, L0 = 0  ->  L = (1-beta) |v|^2 u u^T ;  X = eps^-1/4 (I - uu^T/|u|^2) + (lam+eps)^-1/4 uu^T/|u|^2
    m, n, beta, eps_rel = 9, 5, 0.95, 1e-6
    u = RNG.standard_normal(m); v = RNG.standard_normal(n)
    L, R = oracle.stats_update(np.outer(u, v), np.zeros((m, m)), np.zeros((n, n)), beta)
    lam1 = (1 - beta) * (u @ u) * (v @ v)
    X, lmax, _ = oracle.inverse_root(L, eps_rel)
    assert math.isclose(lmax, lam1, rel_tol=1e-13)
    eps = eps_rel * lam1
    uu = np.outer(u, u) / (u @ u)
    Xref = eps ** -0.25 * (np.eye(m) - uu) + (lam1 + eps) ** -0.25 * uu
    assert relF(X, Xref) < 1e-10


@pytest.mark.parametrize("n,kappa", [(16, 1e2), (64, 1e6), (96, 1e8)])
def test_inverse_root_invariants(n, kappa):
    U = haar(n, RNG)
    d = np.logspace(0, -math.log10(kappa), n)
    A = (U * d) @ U.T
    A = 0.5 * (A + A.T)
    eps_rel = 1.0 / kappa
    X, lmax, _ = oracle.inverse_root(A, eps_rel)
    B = A + eps_rel * lmax * np.eye(n)
    X2 = X @ X
    # the float64 products of this check themselves lose ~kappa * 2^-53
    assert np.linalg.norm(X2 @ X2 @ B - np.eye(n)) / math.sqrt(n) < max(1e-14 * kappa, 1e-12)
    assert np.array_equal(X, X.T) or np.abs(X - X.T).max() < 1e-13 * np.abs(X).max()
    assert np.linalg.norm(X @ A - A @ X) < 1e-12 * np.linalg.norm(X) * np.linalg.norm(A)
    assert np.all(np.linalg.eigvalsh(X) > 0)


def test_inverse_root_4x4_multiprecision_bruteforce():
    # (A + eps I)^(-1/4) by two Denman-Beavers square roots and one inverse at 50 digits
    mpmath.mp.dps = 50
    for seed in range(3):
        rng = np.random.default_rng(100 + seed)
        B = rng.standard_normal((4, 4))
        A = B @ B.T
        eps_rel = 1e-6
        X, lmax, _ = oracle.inverse_root(A, eps_rel)
        Am = mpmath.matrix(A.tolist())
        lam_mp = mpmath.eigsy(Am, eigvals_only=True)
        lmax_mp = max(lam_mp)
        assert abs(lmax - float(lmax_mp)) <= 1e-14 * lmax
        Bm = Am + mpmath.mpf(eps_rel) * lmax_mp * mpmath.eye(4)
        root4 = mpmath.sqrtm(mpmath.sqrtm(Bm))
        Xm = mpmath.inverse(root4)
        Xref = np.array([[float(Xm[i, j]) for j in range(4)] for i in range(4)])
        assert relF(X, Xref) < 1e-12


def test_inverse_root_reports_not_pd_without_clamping():
    A = np.diag([1.0, -1e-3, 0.5])
    st, X, lmax, lam = oracle.inverse_root(A, 1e-6, return_status=True)
    assert st == oracle.NOT_PD and lmax == 1.0
    st, X, _, _ = oracle.inverse_root(A, 1e-2, return_status=True)     # eps = 1e-2 > 1e-3: PD again
    assert st == oracle.OK
    assert np.allclose(np.diag(X), (np.array([1.0, -1e-3, 0.5]) + 1e-2) ** -0.25)


def test_inverse_root_batch_matches_single():
    As = []
    for n in (5, 12, 8):
        B = RNG.standard_normal((n, n)); As.append(B @ B.T)
    Xs, lmax, status = oracle.inverse_root_batch(As, 1e-6)
    assert np.all(status == oracle.OK)
    for A, X, lm in zip(As, Xs, lmax):
        X1, lm1, _ = oracle.inverse_root(A, 1e-6)
        assert np.array_equal(X, X1) and lm == lm1


# ----------------------------------------------------------------------------- precondition

def test_precondition_hand_computed_order_of_factors():
    XL = np.array([[1.0, 2.0], [3.0, 4.0]])
    G = np.array([[0.0, 1.0], [1.0, 0.0]])
    XR = np.array([[1.0, 0.0], [1.0, 1.0]])
    assert np.array_equal(oracle.precondition(XL, G, XR), np.array([[3.0, 1.0], [7.0, 3.0]]))


def test_precondition_identity_and_diagonal_scaling_nonsquare():
    m, n = 5, 8
    G = RNG.standard_normal((m, n))
    assert np.array_equal(oracle.precondition(np.eye(m), G, np.eye(n)), G)
    a = RNG.uniform(0.5, 2, m); b = RNG.uniform(0.5, 2, n)
    P = oracle.precondition(np.diag(a), G, np.diag(b))
    assert np.allclose(P, a[:, None] * G * b[None, :], rtol=1e-15, atol=0)


def test_precondition_whitens_gradient_with_its_own_statistics():
    # L = (1-beta) G G^T, R = (1-beta) G^T G, eps -> 0:  P = (1-beta)^-1/2 U V^T  (G = U S V^T)
    n, beta = 8, 0.95
    G = RNG.standard_normal((n, n))
    L, R = oracle.stats_update(G, np.zeros((n, n)), np.zeros((n, n)), beta)
    XL, _, _ = oracle.inverse_root(L, 1e-12)
    XR, _, _ = oracle.inverse_root(R, 1e-12)
    P = oracle.precondition(XL, G, XR)
    U, s, Vt = np.linalg.svd(G)
    assert relF(P, (1 - beta) ** -0.5 * U @ Vt) < 1e-6 * (s.max() / s.min()) ** 2


# ----------------------------------------------------------------------------- Householder QR / SOAP refresh

def test_householder_qr_hand_computed_2x2():
    Q, R = oracle.householder_qr(np.array([[3.0, 1.0], [4.0, 2.0]]))
    assert np.allclose(Q, [[0.6, -0.8], [0.8, 0.6]], atol=1e-15)
    assert np.allclose(R, [[5.0, 2.2], [0.0, 0.4]], atol=1e-15)


@pytest.mark.parametrize("n", [1, 2, 9, 40])
def test_householder_qr_invariants_and_witness(n):
    Z = RNG.standard_normal((n, n))
    Q, R = oracle.householder_qr(Z)
    assert np.linalg.norm(Q.T @ Q - np.eye(n)) < 1e-13 * n
    assert np.linalg.norm(Q @ R - Z) < 1e-13 * np.linalg.norm(Z) * n
    assert np.all(np.diag(R) >= 0) and np.array_equal(R, np.triu(R))
    q, r = np.linalg.qr(Z)
    s = np.sign(np.diag(r))
    assert np.allclose(Q, q * s, atol=1e-11) and np.allclose(R, r * s[:, None], atol=1e-11)


def test_soap_refresh_diagonal_and_exact_eigenbasis_are_fixed_points():
    d = np.array([3.0, 2.0, 1.0, 0.5])
    Q, R = oracle.soap_refresh(np.diag(d), np.eye(4))
    assert np.array_equal(Q, np.eye(4)) and np.allclose(np.diag(R), d)
    n = 12
    Qs = haar(n, RNG)
    lam = np.linspace(2.0, 0.1, n)
    A = (Qs * lam) @ Qs.T
    Q, R = oracle.soap_refresh(A, Qs)
    assert np.allclose(Q, Qs, atol=1e-13)
    assert np.allclose(R, np.diag(lam), atol=1e-13)


def test_soap_refresh_is_qr_of_power_iteration_and_converges_to_eigenvectors():
    n = 24
    U = haar(n, RNG)
    lam = 2.0 ** -np.arange(n)          # well separated
    A = (U * lam) @ U.T
    Q0 = haar(n, RNG)
    Q, R = oracle.soap_refresh(A, Q0)
    assert np.linalg.norm(Q @ R - A @ Q0) < 1e-13 * np.linalg.norm(A @ Q0)
    assert np.linalg.norm(Q.T @ Q - np.eye(n)) < 1e-13 * n
    for _ in range(40):
        Q, R = oracle.soap_refresh(A, Q)
    lamJ, VJ, _ = oracle.jacobi_eigh(A)
    order = np.argsort(-lamJ)
    for k in range(6):
        assert abs(abs(Q[:, k] @ VJ[:, order[k]]) - 1) < 1e-9
        assert math.isclose(R[k, k], lam[k], rel_tol=1e-9)


# ----------------------------------------------------------------------------- SOAP step

def test_soap_step_identity_bases_is_textbook_adam():
    G = np.array([[0.5, -2.0, 0.0], [1e-3, 4.0, -0.25]])
    m, n = G.shape
    b1, b2, eps = 0.9, 0.95, 1e-8
    N, M, V = oracle.soap_step(G, np.eye(m), np.eye(n), np.zeros((m, n)), np.zeros((m, n)), b1, b2, eps, 1)
    assert np.allclose(M, 0.1 * G, rtol=1e-15) and np.allclose(V, 0.05 * G * G, rtol=1e-15)
    assert np.allclose(N, G / (np.abs(G) + eps), rtol=1e-12, atol=0)
    # second step, hand-derived scalars for entry (0,0): g1 = 0.5, g2 = -1
    G2 = G.copy(); G2[0, 0] = -1.0
    N2, M2, V2 = oracle.soap_step(G2, np.eye(m), np.eye(n), M, V, b1, b2, eps, 2)
    m2 = 0.9 * 0.05 + 0.1 * -1.0            # -0.055
    v2 = 0.95 * 0.0125 + 0.05 * 1.0         # 0.061875
    expect = (m2 / (1 - 0.81)) / (math.sqrt(v2 / (1 - 0.9025)) + eps)
    assert math.isclose(M2[0, 0], m2, rel_tol=1e-14) and math.isclose(V2[0, 0], v2, rel_tol=1e-14)
    assert math.isclose(N2[0, 0], expect, rel_tol=1e-13)


def test_soap_step_gradient_diagonal_in_the_bases_closed_form():
    # G = Q_L D Q_R^T with D "diagonal" (m x n): G' = D, N' = sign(D) on the diagonal, 0 elsewhere.
    m, n = 5, 7
    QL, QR = haar(m, RNG), haar(n, RNG)
    D = np.zeros((m, n))
    dvals = np.array([3.0, -2.0, 1.0, -0.5, 0.25])
    D[np.arange(m), np.arange(m)] = dvals
    G = QL @ D @ QR.T
    N, M, V = oracle.soap_step(G, QL, QR, np.zeros((m, n)), np.zeros((m, n)), 0.9, 0.95, 1e-30, 1)
    S = np.zeros((m, n)); S[np.arange(m), np.arange(m)] = np.sign(dvals)
    # off-diagonal G' entries are rounding noise ~1e-16 and eps=1e-30 would blow them up to O(1):
    # compare moments (well conditioned) and N only through a dense second case below
    assert np.allclose(M, 0.1 * D, atol=1e-15) and np.allclose(V, 0.05 * D * D, atol=1e-15)
    N, _, _ = oracle.soap_step(G, QL, QR, np.zeros((m, n)), np.zeros((m, n)), 0.9, 0.95, 1e-8, 1)
    assert np.allclose(N, QL @ S @ QR.T, atol=1e-6)


def test_soap_step_column_sign_flip_invariance():
    m, n = 6, 4
    QL, QR = haar(m, RNG), haar(n, RNG)
    G = RNG.standard_normal((m, n))
    M0 = 0.1 * RNG.standard_normal((m, n)); V0 = RNG.uniform(0.01, 1, (m, n))
    N, M, V = oracle.soap_step(G, QL, QR, M0, V0, 0.9, 0.95, 1e-8, 3)
    sl = np.array([1, -1, 1, 1, -1, -1.0]); sr = np.array([-1, 1, 1, -1.0])
    Nf, Mf, Vf = oracle.soap_step(G, QL * sl, QR * sr, M0 * np.outer(sl, sr), V0, 0.9, 0.95, 1e-8, 3)
    assert np.allclose(N, Nf, atol=1e-13)
    assert np.allclose(Mf, M * np.outer(sl, sr), atol=1e-15) and np.allclose(Vf, V, atol=1e-15)


# ----------------------------------------------------------------------------- SOAP column order and re-projection

def test_soap_sort_orders_columns_by_estimated_eigenvalue_hand_example():
    # A = diag(2, 5, 3, 5), Q = I: estimates (2, 5, 3, 5) -> order 1, 3 (tie: lower index first), 2, 0
    A = np.diag([2.0, 5.0, 3.0, 5.0])
    Qs, perm, est = oracle.soap_sort(A, np.eye(4))
    assert perm.tolist() == [1, 3, 2, 0] and est.tolist() == [2.0, 5.0, 3.0, 5.0]
    assert np.array_equal(Qs, np.eye(4)[:, [1, 3, 2, 0]])
    # a rotated basis: estimates are Rayleigh quotients q_i^T A q_i, written out by hand for a 2 x 2
    c, s = 0.6, 0.8
    Q = np.array([[c, -s], [s, c]])
    A = np.array([[1.0, 2.0], [2.0, 3.0]])
    r0 = c * c * 1 + 2 * c * s * 2 + s * s * 3            # 0.36 + 1.92 + 1.92
    r1 = s * s * 1 - 2 * c * s * 2 + c * c * 3            # 0.64 - 1.92 + 1.08
    Qs, perm, est = oracle.soap_sort(A, Q)
    assert math.isclose(est[0], r0, rel_tol=1e-15) and math.isclose(est[1], r1, abs_tol=1e-15)
    assert perm.tolist() == [0, 1] and np.array_equal(Qs, Q)
    Qs, perm, _ = oracle.soap_sort(A, Q[:, ::-1].copy())
    assert perm.tolist() == [1, 0] and np.array_equal(Qs, Q)


def test_soap_sort_is_a_permutation_with_non_increasing_estimates_and_matches_the_eigen_order_at_a_fixed_point():
    n = 9
    Qt = haar(n, RNG)
    lam = np.array([0.3, 7.0, 1.5, 1.5, 0.01, 4.0, 2.0, 9.0, 0.7])
    A = (Qt * lam) @ Qt.T
    Qs, perm, est = oracle.soap_sort(A, Qt)
    assert sorted(perm.tolist()) == list(range(n))
    assert np.allclose(est, lam, atol=1e-13)                       # exact eigenvectors: the estimates are the eigenvalues
    assert np.all(np.diff(est[perm]) <= 1e-13)
    big = [i for i in perm if lam[i] not in (1.5,)]
    assert [lam[i] for i in big] == sorted([l for l in lam if l != 1.5], reverse=True)
    assert np.array_equal(Qs, Qt[:, perm])
    # sorting then refreshing leaves an eigenbasis an eigenbasis, now in decreasing order of eigenvalue
    Qr, R = oracle.soap_refresh(A, Qs)
    simple = [k for k in range(n) if lam[perm[k]] != 1.5]                        # the degenerate pair may rotate
    assert np.allclose(np.abs(np.diag(Qr.T @ Qs))[simple], 1.0, atol=1e-9)
    assert np.allclose(np.diag(R), lam[perm], atol=1e-12)


def test_soap_reproject_closed_forms():
    m, n = 5, 4
    QLo, QRo, QLn, QRn = haar(m, RNG), haar(n, RNG), haar(m, RNG), haar(n, RNG)
    M = RNG.standard_normal((m, n))
    # same bases: nothing changes
    assert np.allclose(oracle.soap_reproject(M, QLo, QRo, QLo, QRo), M, atol=1e-14)
    # the matrix the moment stands for in the original space does not change
    M2 = oracle.soap_reproject(M, QLo, QRo, QLn, QRn)
    assert np.allclose(QLn @ M2 @ QRn.T, QLo @ M @ QRo.T, atol=1e-14)
    # and back again
    assert np.allclose(oracle.soap_reproject(M2, QLn, QRn, QLo, QRo), M, atol=1e-13)
    # new bases = old bases with permuted, sign-flipped columns: rows / columns of M follow
    pl, pr = np.array([2, 0, 4, 1, 3]), np.array([3, 1, 0, 2])
    sl, sr = np.array([1, -1, 1, -1, -1.0]), np.array([-1, 1, 1, -1.0])
    M3 = oracle.soap_reproject(M, QLo, QRo, QLo[:, pl] * sl, QRo[:, pr] * sr)
    assert np.allclose(M3, (M[pl][:, pr]) * np.outer(sl, sr), atol=1e-14)
    # hand example, 2 x 2 rotation on the left only: M'' = G(theta)^T M
    c, s = 0.6, 0.8
    G = np.array([[c, -s], [s, c]])
    Mh = np.array([[1.0, 2.0], [3.0, 4.0]])
    exp = np.array([[c * 1 + s * 3, c * 2 + s * 4], [-s * 1 + c * 3, -s * 2 + c * 4]])
    assert np.allclose(oracle.soap_reproject(Mh, np.eye(2), np.eye(2), G, np.eye(2)), exp, atol=1e-15)
    # transposed operand mistakes show on a non-square block with a non-symmetric right rotation
    Gr = np.array([[c, -s, 0], [s, c, 0], [0, 0, 1.0]])
    Mr = np.arange(6.0).reshape(2, 3)
    assert np.allclose(oracle.soap_reproject(Mr, np.eye(2), np.eye(3), np.eye(2), Gr), Mr @ Gr, atol=1e-15)
    assert not np.allclose(Mr @ Gr, Mr @ Gr.T)


def test_soap_step_after_reprojection_continues_the_same_trajectory_in_the_original_space():
    # Adam's first moment is linear in the gradients: carried through a change of bases by
    # re-projection it equals the moment accumulated entirely in the new bases
    m, n = 4, 6
    QLo, QRo, QLn, QRn = haar(m, RNG), haar(n, RNG), haar(m, RNG), haar(n, RNG)
    G1, G2 = RNG.standard_normal((m, n)), RNG.standard_normal((m, n))
    z = np.zeros((m, n))
    _, M1o, _ = oracle.soap_step(G1, QLo, QRo, z, z, 0.9, 0.95, 1e-8, 1)
    Mre = oracle.soap_reproject(M1o, QLo, QRo, QLn, QRn)
    _, M2, _ = oracle.soap_step(G2, QLn, QRn, Mre, z, 0.9, 0.95, 1e-8, 2)
    _, M1n, _ = oracle.soap_step(G1, QLn, QRn, z, z, 0.9, 0.95, 1e-8, 1)
    _, M2n, _ = oracle.soap_step(G2, QLn, QRn, M1n, z, 0.9, 0.95, 1e-8, 2)
    assert np.allclose(M2, M2n, atol=1e-14)
