"""Comparison helpers for the tests (no method arithmetic; plain linear algebra
on results)."""
import numpy as np


def sin_principal_angles(V_ref: np.ndarray, V_test: np.ndarray) -> np.ndarray:
    """Sines of the principal angles between the column spaces, computed as the
    singular values of (I - P_ref) V_test with both bases orthonormalised
    (accurate for small angles, unlike the arccos of the cosines)."""
    A = np.linalg.qr(np.asarray(V_ref, dtype=np.float64))[0]
    B = np.linalg.qr(np.asarray(V_test, dtype=np.float64))[0]
    R = B - A @ (A.T @ B)
    return np.linalg.svd(R, compute_uv=False)


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def reduced_tridiagonal(U: np.ndarray, lam: np.ndarray, shift: float, v1: np.ndarray):
    """Independent route to the Lanczos tridiagonal of H = U diag(lam) U^T + shift I
    started from v1: the Krylov space lives in span([U, v1]), so H restricted to
    an orthonormal basis of that (r+1)-dimensional space is a small dense matrix
    M; a Householder reflector moves the start vector to e_1 and LAPACK's
    Householder reduction to Hessenberg form (tridiagonal, M being symmetric)
    yields the same matrix the Lanczos recurrence builds, up to the signs of the
    off-diagonal.  Returns (diag, |offdiag|)."""
    import scipy.linalg as sla
    U64 = np.asarray(U, dtype=np.float64)
    v = np.asarray(v1, dtype=np.float64)
    v = v / np.linalg.norm(v)
    Bs = np.linalg.qr(np.column_stack([U64, v]))[0]
    G = Bs.T @ U64
    M = G @ np.diag(np.asarray(lam, dtype=np.float64)) @ G.T + float(shift) * np.eye(Bs.shape[1])
    z = Bs.T @ v
    z /= np.linalg.norm(z)
    e1 = np.zeros_like(z)
    e1[0] = 1.0
    u = z - e1
    P = np.eye(len(z)) - 2.0 * np.outer(u, u) / (u @ u) if np.linalg.norm(u) > 0 else np.eye(len(z))
    Hh = sla.hessenberg(P.T @ M @ P)
    return np.diag(Hh).copy(), np.abs(np.diag(Hh, -1))


def reduced_tridiagonal_from_gram(G: np.ndarray, lam: np.ndarray, shift: float):
    """Same independent route as `reduced_tridiagonal`, for sizes where [U, v1]
    cannot be factorised on the host: only its (r+1) x (r+1) Gram matrix G is
    needed.  With [U, v1] = Bs R (R from the Cholesky factor of G), Bs^T U is the
    first r columns of R and Bs^T v1 its last column."""
    import scipy.linalg as sla
    r = G.shape[0] - 1
    R = np.linalg.cholesky(G).T
    Ru = R[:, :r]
    M = Ru @ np.diag(np.asarray(lam, dtype=np.float64)) @ Ru.T + float(shift) * np.eye(r + 1)
    z = R[:, r] / np.linalg.norm(R[:, r])
    e1 = np.zeros_like(z)
    e1[0] = 1.0
    u = z - e1
    P = np.eye(len(z)) - 2.0 * np.outer(u, u) / (u @ u) if np.linalg.norm(u) > 0 else np.eye(len(z))
    Hh = sla.hessenberg(P.T @ M @ P)
    return np.diag(Hh).copy(), np.abs(np.diag(Hh, -1))


def reduced_ritz_coefficients(G: np.ndarray, lam: np.ndarray, shift: float, m: int, k: int, l: int):
    """Reference Ritz pairs of the planted operator expressed in the basis [U, v1]: returns (evals, Cmat)
    with V_ref = [U, v1] @ Cmat, from the same Householder route as `reduced_tridiagonal_from_gram` (the
    Lanczos vectors of the restricted problem are the leading columns of the accumulated reflectors).
    Everything is (r+1)-dimensional float64 work, so it is available at any n."""
    import scipy.linalg as sla
    r = G.shape[0] - 1
    R = np.linalg.cholesky(G).T
    Ru = R[:, :r]
    M = Ru @ np.diag(np.asarray(lam, dtype=np.float64)) @ Ru.T + float(shift) * np.eye(r + 1)
    z = R[:, r] / np.linalg.norm(R[:, r])
    e1 = np.zeros_like(z)
    e1[0] = 1.0
    u = z - e1
    P = np.eye(len(z)) - 2.0 * np.outer(u, u) / (u @ u) if np.linalg.norm(u) > 0 else np.eye(len(z))
    Hh, Qh = sla.hessenberg(P.T @ M @ P, calc_q=True)
    T = Hh[:m, :m]
    T = np.triu(np.tril(T, 1), -1)
    T = 0.5 * (T + T.T)
    ev, S = np.linalg.eigh(T)
    sel = np.concatenate([np.arange(m - 1, m - 1 - k, -1), np.arange(l)]).astype(int)
    Qred = P @ Qh[:, :m]                      # Lanczos vectors of the restricted problem
    Cmat = np.linalg.solve(R, Qred @ S[:, sel])
    resid = abs(Hh[m, m - 1]) * np.abs(S[m - 1, sel]) if Hh.shape[0] > m else np.zeros(len(sel))
    return ev[sel], Cmat, resid, ev
