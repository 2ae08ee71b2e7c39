"""Algorithm 1 (Lanczos with full Gram-Schmidt orthogonalisation) and its
row-sharded form (Algorithm 2), float64.  Test infrastructure only.

Notation: the paper's D (n x m, orthonormal columns) is `Q` here and its
tridiagonal B is held as a band: `alpha` (B[i,i]) and `beta`
(B[i+1,i] = B[i,i+1]).

How the code is organised.  One trip of the algorithm is "apply the operator
to the newest column, remove from the result its components along every column
built so far, normalise what is left and append it".  The only places where
the rows of D meet are inner products, so the driver takes the two reductions
(`inner`: D^T h, `sqnorm`: ||h||^2) as arguments: the single-device algorithm
passes the plain ones, the row-sharded algorithm passes sums of per-block
partial results (its all-reduces), and both share everything else.

Readings of points the paper leaves open (all listed in the design notes):
  * Algorithm 1 writes column m+1 of D and entry B[m+1,m] in its last trip while
    declaring D with m columns: Q gets m+1 columns, B stays m x m, and the last
    beta is kept as the residual norm.
  * The Gram-Schmidt line subtracts the projections onto *all* columns filled
    so far (columns that are still zero contribute nothing).  `passes` repeats
    that line; the diagonal entry is then the sum of the coefficients removed
    along the current column (Eq. 5 names the first of them; the later ones
    vanish in exact arithmetic).
  * Breakdown (the new direction vanishes because the Krylov space is
    exhausted) is not mentioned: the iteration stops when
    ||h after orthogonalisation|| <= breakdown_tol * ||H v_i||, and B is the
    leading m_eff x m_eff block.  The default 1e-6 sits between the ratios of
    healthy steps (0.1 and above on the workloads here) and what rounding leaves
    at an exhausted Krylov space (about 1e-8 in float64 after the error of the
    recurrence has been amplified over some thirty steps).
  * v_1 is handed in (a seeded Gaussian vector) and normalised here.
  * The paper does not state the precision in which D is kept.  `storage`
    (None = float64) names the format of the *stored* vectors: with
    `storage=numpy.float32` every vector the algorithm writes to memory -- the
    operator's output h and each new column of D -- is rounded to that format
    once, while all arithmetic stays float64.  This is what a device
    implementation with fp32 vectors and wide accumulators does, and it is how
    the tests find out which deviations from the float64 run belong to the
    storage format rather than to a particular kernel.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Optional

import numpy as np


@dataclass
class LanczosResult:
    Q: np.ndarray        # n x (m+1) float64; columns 0..m_eff-1 span the Krylov space
    alpha: np.ndarray    # m float64, first m_eff valid
    beta: np.ndarray     # m float64; beta[i] couples columns i and i+1; beta[m_eff-1] = residual norm
    m_eff: int
    hnorm: np.ndarray    # m float64, ||H v_i|| (used by the breakdown rule)


def _stored_as(storage) -> Callable[[np.ndarray], np.ndarray]:
    """What writing a vector to memory does to it: nothing (float64), or one rounding to `storage`."""
    if storage is None or np.dtype(storage) == np.float64:
        return lambda x: x
    fmt = np.dtype(storage)
    return lambda x: np.asarray(x, dtype=np.float64).astype(fmt).astype(np.float64)


def _remove_components(filled: np.ndarray, h: np.ndarray, inner) -> tuple:
    """The Gram-Schmidt line once: h minus its projections onto the columns of `filled`.
    Returns (new h, coefficient that was removed along the last column)."""
    coeff = inner(filled, h)                      # D^T h
    return h - filled @ coeff, coeff[-1]


def _run(hvp, v1: np.ndarray, m: int, passes: int, breakdown_tol: float, storage, inner, sqnorm) -> LanczosResult:
    keep = _stored_as(storage)
    v1 = np.asarray(v1, dtype=np.float64)
    n = v1.shape[0]
    Q = np.zeros((n, m + 1), order="F")
    band = np.zeros((2, m))                       # row 0: diagonal of B, row 1: its off-diagonal
    hnorm = np.zeros(m)
    Q[:, 0] = keep(v1 / np.sqrt(sqnorm(v1)))      # first column: the normalised random vector
    m_eff = m
    for i in range(m):
        h = keep(np.asarray(hvp(Q[:, i]), dtype=np.float64))
        hnorm[i] = np.sqrt(sqnorm(h))
        for _ in range(passes):                   # against all filled columns; Eq. 5: the part along v_i is B[i,i]
            h, along_current = _remove_components(Q[:, : i + 1], h, inner)
            band[0, i] += along_current
        band[1, i] = np.sqrt(sqnorm(h))           # B[i+1,i] = B[i,i+1] (Eq. 6)
        if not band[1, i] > breakdown_tol * hnorm[i]:
            m_eff = i + 1
            break
        Q[:, i + 1] = keep(h / band[1, i])
    return LanczosResult(Q=Q, alpha=band[0], beta=band[1], m_eff=m_eff, hnorm=hnorm)


def lanczos(hvp: Callable[[np.ndarray], np.ndarray], v1: np.ndarray, m: int,
            passes: int = 1, breakdown_tol: float = 1e-6, storage: Optional[type] = None) -> LanczosResult:
    """Algorithm 1 on one device: the reductions are the plain ones."""
    return _run(hvp, v1, m, passes, breakdown_tol, storage,
                inner=lambda D, h: D.T @ h, sqnorm=lambda h: float(h @ h))


def tridiagonal(alpha: np.ndarray, beta: np.ndarray, m_eff: int) -> np.ndarray:
    """The dense m_eff x m_eff matrix B of Algorithm 1."""
    B = np.diag(np.asarray(alpha[:m_eff], dtype=np.float64))
    if m_eff > 1:
        off = np.asarray(beta[: m_eff - 1], dtype=np.float64)
        B += np.diag(off, 1) + np.diag(off, -1)
    return B


def row_blocks(n: int, C: int) -> list:
    """C contiguous row ranges [s_c, e_c) covering 0..n (the virtual devices of Algorithm 2)."""
    edges = np.linspace(0, n, C + 1).astype(int)
    return [slice(int(edges[c]), int(edges[c + 1])) for c in range(C)]


def lanczos_row_sharded(hvp: Callable[[np.ndarray], np.ndarray], v1: np.ndarray, m: int, C: int,
                        passes: int = 1, breakdown_tol: float = 1e-6, storage: Optional[type] = None) -> LanczosResult:
    """Algorithm 2 emulated in one process: C virtual devices each own a
    contiguous row block of D and of h.  A device can only form the part of an
    inner product that its own rows contribute; the all-reduce of the algorithm
    adds those parts, device 0 first.  The operator sees the whole current
    vector (the algorithm's all-gather is the identity in one address space).
    Same result structure as `lanczos`."""
    blocks = row_blocks(np.asarray(v1).shape[0], C)

    def all_reduced_inner(D, h):
        partial = [D[b].T @ h[b] for b in blocks]            # what each device computes from its rows
        return np.sum(partial, axis=0)                       # all-reduce

    def all_reduced_sqnorm(h):
        return float(sum(float(h[b] @ h[b]) for b in blocks))  # all-reduce of the local squared norms

    return _run(hvp, v1, m, passes, breakdown_tol, storage, inner=all_reduced_inner, sqnorm=all_reduced_sqnorm)
