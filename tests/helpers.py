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


# ---------------------------------------------------------------------------------------------------
# What fp32 storage of the Krylov basis does to the Ritz pairs (CPU emulation with the oracle)
# ---------------------------------------------------------------------------------------------------

def reduced_problem(G: np.ndarray, lam: np.ndarray, shift: float):
    """The planted operator restricted to span([U, v1]), from the Gram matrix G of [U, v1] alone: with
    [U, v1] = Bs R (R the transposed Cholesky factor of G, Bs orthonormal) the operator acts on Bs-coordinates as
    M + shift I, M = R_u diag(lam) R_u^T, and the start vector is the normalised last column of R.
    Returns (M, z, R)."""
    r = G.shape[0] - 1
    R = np.linalg.cholesky(np.asarray(G, dtype=np.float64)).T
    Ru = R[:, :r]
    M = Ru @ np.diag(np.asarray(lam, dtype=np.float64)) @ Ru.T
    z = R[:, r] / np.linalg.norm(R[:, r])
    return M, z, R


def planted_embedding(M: np.ndarray, z: np.ndarray, n_rows: int, seed: int):
    """An n_rows-row planted operator U' diag(lam') U'^T (+ shift I) and a start vector whose restriction to
    span([U', v1']) is exactly (M, z): a seeded random orthonormal basis Bo carries the small problem into
    n_rows dimensions.  Two embeddings of the same (M, z) produce the same tridiagonal in exact arithmetic; they
    differ in how their vectors round.  Returns (U', lam', v1', Bo)."""
    d = M.shape[0]
    rng = np.random.default_rng([250500982, 77, int(seed)])
    Bo = np.linalg.qr(rng.standard_normal((int(n_rows), d)))[0]
    ev, W = np.linalg.eigh(M)
    keep = np.argsort(-np.abs(ev))[: d - 1]            # M has rank d - 1: drop its (numerically) zero eigenvalue
    return Bo @ W[:, keep], ev[keep], Bo @ z, Bo


def _sines(A_ref: np.ndarray, B_test: np.ndarray) -> np.ndarray:
    A = np.linalg.qr(A_ref)[0]
    B = np.linalg.qr(B_test)[0]
    return np.linalg.svd(B - A @ (A.T @ B), compute_uv=False)


def storage_emulation(G: np.ndarray, lam: np.ndarray, shift: float, m: int, k: int, l: int,
                      n_rows: int = 1 << 16, seed: int = 0, storage=np.float32, passes: int = 2) -> dict:
    """Runs the oracle's Lanczos recurrence and Ritz extraction twice on one n_rows-row embedding of the planted
    problem described by (G, lam, shift): once with float64 vectors and once with every stored vector (operator
    output, new basis column) rounded to `storage` while the arithmetic stays float64.  The differences between
    the two runs are what the storage format alone costs.  Per requested pair (k largest descending, then l
    smallest ascending):
        value_abs_err   |theta_storage - theta_float64|
        out_norm        norm of the storage run's Ritz vector outside span([U, v1]) -- directions in the
                        eigenspace of `shift`, which rounding feeds into the Krylov space
        in_span_leave   how far the in-span part of that Ritz vector leaves the float64 run's block (top or
                        bottom) of Ritz vectors
    and per block the largest principal-angle sine, once for the whole vectors (`total_sin`) and once for their
    in-span parts (`in_span_sin`); `dT[i]` = max(|d alpha_i|, |d beta_i|); `qtq` = max |Q^T Q - I| of the
    storage run; `resid` = the float64 run's residual estimates, `evals` its Ritz values."""
    import oracle
    M, z, _ = reduced_problem(G, lam, shift)
    U, lam_e, v1, Bo = planted_embedding(M, z, n_rows, seed)
    op = lambda v: oracle.hvp_planted(U, lam_e, float(shift), v)
    runs = {}
    for name, fmt in (("float64", None), ("storage", storage)):
        res = oracle.lanczos(op, v1, m, passes=passes, storage=fmt)
        assert res.m_eff == m, "the emulation expects a run without breakdown"
        runs[name] = (res, oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, k, l))
    (r64, z64), (rst, zst) = runs["float64"], runs["storage"]
    if storage is not None:                                   # the Ritz vectors are stored in the same format
        zst.V = zst.V.astype(storage).astype(np.float64)
    Y = Bo.T @ zst.V                                          # in-span coordinates of the storage run's Ritz vectors
    out = zst.V - Bo @ Y
    out_norm = np.linalg.norm(out, axis=0)
    Cref = Bo.T @ z64.V
    blocks = {"top": slice(0, k), "bottom": slice(k, k + l)}
    total_sin, in_span_sin = {}, {}
    in_span_leave = np.zeros(k + l)
    for name, blk in blocks.items():
        if blk.stop == blk.start:
            continue
        total_sin[name] = float(_sines(z64.V[:, blk], zst.V[:, blk]).max())
        in_span_sin[name] = float(_sines(Cref[:, blk], Y[:, blk]).max())
        A = np.linalg.qr(Cref[:, blk])[0]
        Yb = Y[:, blk] / np.linalg.norm(Y[:, blk], axis=0)
        in_span_leave[blk] = np.linalg.norm(Yb - A @ (A.T @ Yb), axis=0)
    Qs = rst.Q[:, :m]
    return dict(evals=z64.evals, resid=z64.resid, value_abs_err=np.abs(zst.evals - z64.evals), out_norm=out_norm,
                in_span_leave=in_span_leave, total_sin=total_sin, in_span_sin=in_span_sin,
                dT=np.maximum(np.abs(rst.alpha - r64.alpha), np.abs(rst.beta - r64.beta)),
                qtq=float(np.abs(Qs.T @ Qs - np.eye(m)).max()),
                alpha=r64.alpha.copy(), beta=r64.beta.copy(), all_evals=z64.all_evals)


def synthetic_gram(r: int, n_true: int, seed: int) -> np.ndarray:
    """Gram matrix of [U, v1] for an exactly orthonormal U (n_true x r) and a Gaussian v1 of n_true entries, drawn
    directly: U^T v1 ~ N(0, I_r) and ||v1||^2 ~ chi^2 with n_true degrees of freedom (~ n_true)."""
    rng = np.random.default_rng([250500982, 78, int(seed)])
    a = rng.standard_normal(r)
    G = np.eye(r + 1)
    G[:r, r] = G[r, :r] = a
    G[r, r] = a @ a + rng.chisquare(n_true - r)
    return G


# ---------------------------------------------------------------------------------------------------
# Algorithm 3 at sizes the numpy oracle cannot hold: the same equations with library float64 operations on
# whatever device the tensors live on, V-hat visited in row chunks.  Pinned against the oracle on the CPU
# (tests/test_oracle_pins.py::test_chunked_float64_state_equals_the_oracle).
# ---------------------------------------------------------------------------------------------------

class Float64State:
    """Full-length float64 copies of (w_a, momentum b, multiplier pi, anchor w) advanced by Eq. 14 (heavy ball as the
    base optimiser, the Newton term in its printed form) and Eq. 11 / Algorithm 3."""

    def __init__(self, w0, chunk: int = 1 << 20):
        import torch
        self.torch = torch
        self.w = w0.double().clone()
        self.b = torch.zeros_like(self.w)
        self.pi = torch.zeros_like(self.w)
        self.anchor = None
        self.chunk = chunk

    def _vt(self, Vm, x):
        """V^T x for V given as its transpose Vm (columns of V are rows of Vm, fp32), x float64."""
        n = x.shape[0]
        out = self.torch.zeros(Vm.shape[0], dtype=self.torch.float64, device=x.device)
        for lo in range(0, n, self.chunk):
            hi = min(n, lo + self.chunk)
            out += Vm[:, lo:hi].double() @ x[lo:hi]
        return out

    def begin(self, sigma: float):
        self.anchor = self.w + self.pi / sigma          # w = w_a + pi / sigma; w_a restarts from it
        self.w = self.anchor.clone()

    def step(self, Vm, evals, g, alpha: float, lr: float, momentum: float, sigma: float, with_pi: bool = True):
        torch = self.torch
        n = self.w.shape[0]
        gt = g.double() + self.pi if with_pi else g.double()
        sig = sigma if with_pi else 0.0
        c = self._vt(Vm, gt)
        # printed form of the Newton term: V^T applied to the projected gradient V (V^T g~)
        in_span = torch.empty_like(gt)
        for lo in range(0, n, self.chunk):
            hi = min(n, lo + self.chunk)
            in_span[lo:hi] = Vm[:, lo:hi].double().T @ c
        c_printed = self._vt(Vm, in_span)
        newton = alpha * c_printed / (torch.as_tensor(evals, dtype=torch.float64, device=gt.device) + sig)
        self.b = momentum * self.b + (gt - in_span)
        o = -lr * self.b
        e = self._vt(Vm, o)
        for lo in range(0, n, self.chunk):
            hi = min(n, lo + self.chunk)
            self.w[lo:hi] += o[lo:hi] - Vm[:, lo:hi].double().T @ (newton + e)

    def end(self, sigma: float):
        self.pi = self.pi + sigma * (self.w - self.anchor)
