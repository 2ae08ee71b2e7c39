"""Curvature operators v -> H v used as the input `hvp_t` of Algorithm 1 (oracle side, float64).

The paper obtains `hvp_t` from a network by automatic differentiation
(Section II-B, the paragraph introducing Algorithm 1).  The synthetic workloads
replace it by operators with a known structure; each is written here as its
definition.  Test infrastructure only.
"""
from __future__ import annotations

import numpy as np


def hvp_planted(U: np.ndarray, lam: np.ndarray, shift: float, v: np.ndarray) -> np.ndarray:
    """H v for H = U diag(lam) U^T + shift I (planted-spectrum workload).

    U (n x r) and lam (r) are taken exactly as stored (fp32 values upcast),
    so this is the same operator the GPU applies."""
    U64 = np.asarray(U, dtype=np.float64)
    v64 = np.asarray(v, dtype=np.float64)
    coeff = U64.T @ v64
    return U64 @ (np.asarray(lam, dtype=np.float64) * coeff) + float(shift) * v64


def hvp_planted_chunked(U: np.ndarray, lam: np.ndarray, shift: float, v: np.ndarray,
                        rows: int = 1 << 20) -> np.ndarray:
    """Same operator, upcasting U one row block at a time (for n where a
    float64 copy of U would not fit in memory)."""
    v64 = np.asarray(v, dtype=np.float64)
    n, r = U.shape
    coeff = np.zeros(r)
    for lo in range(0, n, rows):
        coeff += np.asarray(U[lo:lo + rows], dtype=np.float64).T @ v64[lo:lo + rows]
    d = np.asarray(lam, dtype=np.float64) * coeff
    out = float(shift) * v64
    for lo in range(0, n, rows):
        out[lo:lo + rows] += np.asarray(U[lo:lo + rows], dtype=np.float64) @ d
    return out


def hvp_diag(d: np.ndarray, v: np.ndarray) -> np.ndarray:
    """H v for H = diag(d)."""
    return np.asarray(d, dtype=np.float64) * np.asarray(v, dtype=np.float64)


def softmax_rows(logits: np.ndarray) -> np.ndarray:
    z = logits - logits.max(axis=1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=1, keepdims=True)


def hvp_softmax_ggn(X: np.ndarray, W: np.ndarray, v: np.ndarray) -> np.ndarray:
    """Generalised Gauss-Newton product of the mean softmax cross-entropy of a
    linear classifier, logits = X W, with respect to W (d x C, flattened
    row-major into a vector of length d*C):

        H v = X^T [ (diag(p_b) - p_b p_b^T) (X V)_b ]_b / B ,   V = v.reshape(d, C),

    where p_b = softmax(x_b^T W) and the bracket acts on each row b.  Because
    the logits are linear in W this equals the exact Hessian of the loss."""
    X64 = np.asarray(X, dtype=np.float64)
    W64 = np.asarray(W, dtype=np.float64)
    B, d = X64.shape
    C = W64.shape[1]
    V = np.asarray(v, dtype=np.float64).reshape(d, C)
    P = softmax_rows(X64 @ W64)
    Z = X64 @ V                                   # directional change of the logits, B x C
    Y = P * Z - P * np.sum(P * Z, axis=1, keepdims=True)
    return (X64.T @ Y / B).reshape(-1)
