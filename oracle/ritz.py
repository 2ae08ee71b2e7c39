"""Ritz extraction: eigendecomposition of the tridiagonal B and the selection of
the k largest and l smallest Ritz pairs (Eq. 8 and the paragraph after it),
float64.  Test infrastructure only.

Readings: the k largest values come first in descending order, then the l
smallest in ascending order; eigenvector signs are whatever the dense solver
returns (callers compare subspaces); the residual estimate of pair j is
beta_last * |last component of its eigenvector of B|.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from .lanczos import tridiagonal


@dataclass
class RitzResult:
    evals: np.ndarray    # k+l float64: k largest (descending) then l smallest (ascending)  -- the paper's a-hat
    V: np.ndarray        # n x (k+l) float64                                                -- the paper's V-hat
    resid: np.ndarray    # k+l residual estimates
    S: np.ndarray        # m_eff x (k+l) selected eigenvectors of B
    all_evals: np.ndarray  # every eigenvalue of B, ascending (the paper's u)


def ritz(Q: np.ndarray, alpha: np.ndarray, beta: np.ndarray, m_eff: int, k: int, l: int) -> RitzResult:
    if k < 0 or l < 0 or k + l < 1 or k + l > m_eff:
        raise ValueError("need 1 <= k + l <= m_eff")
    B = tridiagonal(alpha, beta, m_eff)
    u, Umat = np.linalg.eigh(B)                           # ascending
    top = np.arange(m_eff - 1, m_eff - 1 - k, -1)        # k largest, descending
    bottom = np.arange(0, l)                              # l smallest, ascending
    sel = np.concatenate([top, bottom]).astype(int)
    S = Umat[:, sel]
    Z_sel = np.asarray(Q[:, :m_eff], dtype=np.float64) @ S    # selected columns of Z = D U
    resid = abs(float(beta[m_eff - 1])) * np.abs(S[m_eff - 1, :])
    return RitzResult(evals=u[sel], V=Z_sel, resid=resid, S=S, all_evals=u)
