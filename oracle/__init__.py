"""Float64 CPU oracle for the Shampoo / SOAP preconditioner pipeline (ctypes view of
``asteria_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py``.  The product package never imports this module and
this module never imports the product package.

Every function takes and returns ``numpy.float64`` arrays (C order).  Inputs that were
produced in bf16 / fp32 are converted exactly (both formats embed in float64).

Paper passages followed: Sec. II-A Eq. 1 (Shampoo update), Eq. 2 (SOAP update); Sec. I and
Sec. III-B (the Kronecker-factor statistics L, R and their inverse factors).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "asteria_oracle.c")
_LIB = os.path.join(_HERE, "libasteria_oracle.so")

OK, NOT_CONVERGED, NOT_PD, BAD_ARG = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        lib.oracle_version.restype = ctypes.c_int
        lib.oracle_stats_update.argtypes = [ctypes.c_int, ctypes.c_int, dp, dp, dp, ctypes.c_double]
        lib.oracle_jacobi_eigh.argtypes = [ctypes.c_int, dp, dp, dp, ctypes.c_double, ctypes.c_int, ip]
        lib.oracle_inverse_root.argtypes = [ctypes.c_int, dp, ctypes.c_int, ctypes.c_int,
                                            ctypes.c_double, dp, dp, dp]
        lib.oracle_inverse_root_batch.argtypes = [ctypes.c_int, ip, ctypes.POINTER(dp), ctypes.c_int,
                                                  ctypes.c_int, dp, ctypes.POINTER(dp), dp, ip]
        lib.oracle_precondition.argtypes = [ctypes.c_int, ctypes.c_int, dp, dp, dp, dp]
        lib.oracle_householder_qr.argtypes = [ctypes.c_int, dp, dp, dp]
        lib.oracle_soap_refresh.argtypes = [ctypes.c_int, dp, dp, dp]
        lib.oracle_soap_step.argtypes = [ctypes.c_int, ctypes.c_int, dp, dp, dp, dp, dp,
                                         ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                         ctypes.c_int, dp]
        lib.oracle_soap_sort.argtypes = [ctypes.c_int, dp, dp, ip, dp]
        lib.oracle_soap_reproject.argtypes = [ctypes.c_int, ctypes.c_int, dp, dp, dp, dp, dp]
        _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


class OracleError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: oracle status {status}")
        self.status = status


def stats_update(G, L, R, beta: float):
    """L' = beta L + (1-beta) G G^T,  R' = beta R + (1-beta) G^T G.  Returns (L', R')."""
    G = _f64(G)
    m, n = G.shape
    L = _f64(L).copy()
    R = _f64(R).copy()
    assert L.shape == (m, m) and R.shape == (n, n)
    st = _load().oracle_stats_update(m, n, _p(G), _p(L), _p(R), float(beta))
    if st != OK:
        raise OracleError(st, "stats_update")
    return L, R


def jacobi_eigh(A, tol: float = 1e-14, max_sweeps: int = 60):
    """Cyclic-Jacobi eigendecomposition.  Returns (lam, V, sweeps); A = V diag(lam) V^T,
    eigenvalues in the order Jacobi leaves them on the diagonal (unsorted)."""
    A = _f64(A)
    n = A.shape[0]
    assert A.shape == (n, n)
    lam = np.empty(n)
    V = np.empty((n, n))
    sweeps = ctypes.c_int(0)
    st = _load().oracle_jacobi_eigh(n, _p(A), _p(lam), _p(V), float(tol), int(max_sweeps),
                                    ctypes.byref(sweeps))
    if st != OK:
        raise OracleError(st, "jacobi_eigh")
    return lam, V, sweeps.value


def inverse_root(A, eps: float, relative: bool = True, p: int = 4, return_status: bool = False):
    """X = (A + eps' I)^(-1/p), eps' = eps * lambda_max(A) if ``relative`` else eps.

    Returns (X, lambda_max, lam).  With ``return_status`` returns (status, X, lambda_max, lam)
    instead of raising when A + eps' I is not positive definite (status NOT_PD)."""
    A = _f64(A)
    n = A.shape[0]
    assert A.shape == (n, n)
    X = np.full((n, n), np.nan)
    lam = np.empty(n)
    lmax = ctypes.c_double(0.0)
    st = _load().oracle_inverse_root(n, _p(A), int(p), 1 if relative else 0, float(eps),
                                     _p(X), ctypes.byref(lmax), _p(lam))
    if return_status:
        return st, X, lmax.value, lam
    if st != OK:
        raise OracleError(st, "inverse_root")
    return X, lmax.value, lam


def inverse_root_batch(As, eps, relative: bool = True, p: int = 4):
    """Independent factors, one OpenMP thread each.  Returns (list of X, lambda_max array,
    status array).  Used to time the oracle on all host cores."""
    As = [_f64(a) for a in As]
    cnt = len(As)
    ns = (ctypes.c_int * cnt)(*[a.shape[0] for a in As])
    Xs = [np.full_like(a, np.nan) for a in As]
    dp = ctypes.POINTER(ctypes.c_double)
    Ap = (dp * cnt)(*[_p(a) for a in As])
    Xp = (dp * cnt)(*[_p(x) for x in Xs])
    epsv = _f64(np.broadcast_to(np.asarray(eps, dtype=np.float64), (cnt,)))
    lmax = np.zeros(cnt)
    status = np.zeros(cnt, dtype=np.intc)
    st = _load().oracle_inverse_root_batch(cnt, ns, Ap, int(p), 1 if relative else 0, _p(epsv), Xp,
                                           _p(lmax), status.ctypes.data_as(ctypes.POINTER(ctypes.c_int)))
    if st != OK:
        raise OracleError(st, "inverse_root_batch")
    return Xs, lmax, status


def precondition(XL, G, XR):
    """P = X_L G X_R (Eq. 1)."""
    XL, G, XR = _f64(XL), _f64(G), _f64(XR)
    m, n = G.shape
    assert XL.shape == (m, m) and XR.shape == (n, n)
    P = np.empty((m, n))
    st = _load().oracle_precondition(m, n, _p(XL), _p(G), _p(XR), _p(P))
    if st != OK:
        raise OracleError(st, "precondition")
    return P


def householder_qr(Z):
    """Householder QR with diag(R) >= 0.  Returns (Q, R)."""
    Z = _f64(Z)
    n = Z.shape[0]
    assert Z.shape == (n, n)
    Q = np.empty((n, n))
    R = np.empty((n, n))
    st = _load().oracle_householder_qr(n, _p(Z), _p(Q), _p(R))
    if st != OK:
        raise OracleError(st, "householder_qr")
    return Q, R


def soap_refresh(A, Q):
    """Q' = qr(A Q).Q with diag(R) >= 0.  Returns (Q', R)."""
    A = _f64(A)
    Q = _f64(Q).copy()
    n = A.shape[0]
    assert A.shape == (n, n) and Q.shape == (n, n)
    R = np.empty((n, n))
    st = _load().oracle_soap_refresh(n, _p(A), _p(Q), _p(R))
    if st != OK:
        raise OracleError(st, "soap_refresh")
    return Q, R


def soap_step(G, QL, QR, M, V, beta1: float, beta2: float, adam_eps: float, t: int):
    """Eq. 2 with Adam in the rotated basis.  Returns (N, M', V')."""
    G, QL, QR = _f64(G), _f64(QL), _f64(QR)
    m, n = G.shape
    M = _f64(M).copy()
    V = _f64(V).copy()
    assert QL.shape == (m, m) and QR.shape == (n, n) and M.shape == (m, n) and V.shape == (m, n)
    N = np.empty((m, n))
    st = _load().oracle_soap_step(m, n, _p(G), _p(QL), _p(QR), _p(M), _p(V), float(beta1),
                                  float(beta2), float(adam_eps), int(t), _p(N))
    if st != OK:
        raise OracleError(st, "soap_step")
    return N, M, V


def soap_sort(A, Q):
    """Columns of Q ordered by decreasing q_i^T A q_i (ties: increasing index).
    Returns (Q[:, perm], perm, est in the old order)."""
    A = _f64(A)
    Q = _f64(Q).copy()
    n = A.shape[0]
    assert A.shape == (n, n) and Q.shape == (n, n)
    perm = np.zeros(n, dtype=np.intc)
    est = np.empty(n)
    st = _load().oracle_soap_sort(n, _p(A), _p(Q), perm.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), _p(est))
    if st != OK:
        raise OracleError(st, "soap_sort")
    return Q, perm.astype(np.int64), est


def soap_reproject(M, QL_old, QR_old, QL_new, QR_new):
    """A moment M held in the bases (QL_old, QR_old) re-expressed in (QL_new, QR_new):
    QL_new^T (QL_old M QR_old^T) QR_new."""
    M = _f64(M).copy()
    m, n = M.shape
    QLo, QRo, QLn, QRn = _f64(QL_old), _f64(QR_old), _f64(QL_new), _f64(QR_new)
    assert QLo.shape == (m, m) == QLn.shape and QRo.shape == (n, n) == QRn.shape
    st = _load().oracle_soap_reproject(m, n, _p(QLo), _p(QRo), _p(QLn), _p(QRn), _p(M))
    if st != OK:
        raise OracleError(st, "soap_reproject")
    return M
