"""Algorithm 1 (Lanczos with full Gram-Schmidt orthogonalisation), float64.

Notation: the paper's D (n x m, orthonormal columns) is `Q` here and its
tridiagonal B is held as the two diagonals `alpha` (B[i,i]) and `beta`
(B[i+1,i] = B[i,i+1]).  Test infrastructure only.

Readings of points the paper leaves open (all listed in the design notes):
  * Algorithm 1 writes column m+1 of D and entry B[m+1,m] in its last trip while
    declaring D with m columns: Q gets m+1 columns, B stays m x m, and the last
    beta is kept as the residual norm.
  * The Gram-Schmidt line subtracts the projections onto *all* columns filled
    so far (columns that are still zero contribute nothing).
  * Breakdown (the new direction vanishes because the Krylov space is
    exhausted) is not mentioned: the iteration stops when
    ||h after orthogonalisation|| <= breakdown_tol * ||H v_i||, and B is the
    leading m_eff x m_eff block.  The default 1e-6 sits between the ratios of
    healthy steps (0.1 and above on the workloads here) and what rounding leaves
    at an exhausted Krylov space (about 1e-8 in float64 after the error of the
    recurrence has been amplified over some thirty steps).
  * v_1 is handed in (a seeded Gaussian vector) and normalised here.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable

import numpy as np


@dataclass
class LanczosResult:
    Q: np.ndarray        # n x (m+1) float64; columns 0..m_eff-1 span the Krylov space
    alpha: np.ndarray    # m float64, first m_eff valid
    beta: np.ndarray     # m float64; beta[i] couples columns i and i+1; beta[m_eff-1] = residual norm
    m_eff: int
    hnorm: np.ndarray    # m float64, ||H v_i|| (used by the breakdown rule)


def lanczos(hvp: Callable[[np.ndarray], np.ndarray], v1: np.ndarray, m: int,
            passes: int = 1, breakdown_tol: float = 1e-6) -> LanczosResult:
    v1 = np.asarray(v1, dtype=np.float64)
    n = v1.shape[0]
    Q = np.zeros((n, m + 1), order="F")
    alpha = np.zeros(m)
    beta = np.zeros(m)
    hnorm = np.zeros(m)
    # initialisation: first column is the normalised random vector
    Q[:, 0] = v1 / np.linalg.norm(v1)
    m_eff = m
    for i in range(m):
        v_i = Q[:, i]
        h = np.asarray(hvp(v_i), dtype=np.float64)
        hnorm[i] = np.linalg.norm(h)
        alpha[i] = h @ v_i                               # B[i,i] (Eq. 5)
        for _ in range(passes):                          # Gram-Schmidt against all filled columns
            D = Q[:, : i + 1]
            h = h - D @ (D.T @ h)
        beta[i] = np.linalg.norm(h)                      # B[i+1,i] = B[i,i+1] (Eq. 6)
        if not beta[i] > breakdown_tol * hnorm[i]:
            m_eff = i + 1
            break
        Q[:, i + 1] = h / beta[i]
    return LanczosResult(Q=Q, alpha=alpha, beta=beta, m_eff=m_eff, hnorm=hnorm)


def tridiagonal(alpha: np.ndarray, beta: np.ndarray, m_eff: int) -> np.ndarray:
    """The dense m_eff x m_eff matrix B of Algorithm 1."""
    B = np.diag(np.asarray(alpha[:m_eff], dtype=np.float64))
    if m_eff > 1:
        off = np.asarray(beta[: m_eff - 1], dtype=np.float64)
        B += np.diag(off, 1) + np.diag(off, -1)
    return B


def lanczos_row_sharded(hvp: Callable[[np.ndarray], np.ndarray], v1: np.ndarray, m: int, C: int,
                        breakdown_tol: float = 1e-6) -> LanczosResult:
    """Algorithm 2 emulated in one process: C virtual devices each own a
    contiguous row block [s_c, e_c) of D and of h.  The collectives become
    plain Python: all_gather = concatenation of the blocks, all_reduce = sum of
    the per-device partial results.  Returns the same structure as `lanczos`,
    with Q assembled from the blocks."""
    v1 = np.asarray(v1, dtype=np.float64)
    n = v1.shape[0]
    edges = np.linspace(0, n, C + 1).astype(int)
    blocks = [slice(edges[c], edges[c + 1]) for c in range(C)]
    v1 = v1 / np.linalg.norm(v1)                        # same seed, same vector on every device
    D = [np.zeros((b.stop - b.start, m + 1)) for b in blocks]
    for c, b in enumerate(blocks):
        D[c][:, 0] = v1[b]
    alpha = np.zeros(m)
    beta = np.zeros(m)
    hnorm = np.zeros(m)
    m_eff = m
    for i in range(m):
        v_i = np.concatenate([D[c][:, i] for c in range(C)])            # all_gather
        h = np.asarray(hvp(v_i), dtype=np.float64)
        hnorm[i] = np.linalg.norm(h)
        alpha[i] = h @ v_i
        mvec = sum(D[c][:, : i + 1].T @ h[b] for c, b in enumerate(blocks))   # all_reduce
        h_loc = [h[b] - D[c][:, : i + 1] @ mvec for c, b in enumerate(blocks)]
        beta[i] = np.sqrt(sum(float(x @ x) for x in h_loc))             # all_reduce
        if not beta[i] > breakdown_tol * hnorm[i]:
            m_eff = i + 1
            break
        for c in range(C):
            D[c][:, i + 1] = h_loc[c] / beta[i]
    return LanczosResult(Q=np.concatenate(D, axis=0), alpha=alpha, beta=beta, m_eff=m_eff, hnorm=hnorm)
