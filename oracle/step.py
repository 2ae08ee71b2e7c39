"""One model update w <- w + Delta_1 + Delta_2 of the hybrid-order optimiser
(Eq. 4 and Eq. 12; with a dual variable pi, Eq. 14), float64.  The base
first-order optimiser is heavy-ball momentum.  Test infrastructure only.

Readings of points the paper leaves open:
  * The base optimiser returns a descent vector (its sign and learning rate
    are inside it, since the update is w + Delta_1 + Delta_2): the buffer is
    b <- momentum * b + x and the returned vector is -lr * b.
  * Eq. 14 names "g_1" inside Delta_2 without saying whether it is the
    projection of g_t or of g_t + pi.  `g1_reading="projected"` (default)
    removes the projection of g_t + pi, mirroring Eq. 12; "literal" removes the
    projection of g_t only.  With V-hat fixed and a linear base optimiser both
    give the same Delta_2.
  * Eq. 4 and Eq. 14 write a plain inverse of A_1 (+ sigma I): `curv_mode =
    "signed"` is that; "abs" divides by |a-hat| + sigma instead.
  * The term sigma (w_a - w) of the gradient of the augmented Lagrangian does
    not appear in Eq. 14 and is not added.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np


def fosi_step(w: np.ndarray, g: np.ndarray, V: np.ndarray, evals: np.ndarray, mom: np.ndarray,
              alpha: float, lr: float, momentum: float, sigma: float = 0.0,
              pi: Optional[np.ndarray] = None, curv_mode: str = "signed",
              g1_reading: str = "projected") -> Tuple[np.ndarray, np.ndarray]:
    """Returns (w_new, mom_new).  V is n x (k+l) with orthonormal columns (may
    have zero columns), evals the matching Ritz values.  Without `pi` this is
    the plain update (sigma is ignored)."""
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    a_hat = np.asarray(evals, dtype=np.float64)
    b = np.asarray(mom, dtype=np.float64)
    if pi is None:
        g_tilde, sig = g, 0.0
    else:
        g_tilde, sig = g + np.asarray(pi, dtype=np.float64), float(sigma)

    # Delta_1: alpha-scaled Newton step inside span(V-hat).  As printed (Eq. 4, Eq. 14) the inverse acts on
    # V^T applied to the projected gradient V (V^T g~), not on V^T g~ itself.
    in_span = V @ (V.T @ g_tilde)
    c = V.T @ in_span
    denom = a_hat + sig if curv_mode == "signed" else np.abs(a_hat) + sig
    delta1 = -alpha * (V @ (c / denom))

    # Delta_2: base optimiser on the complement, re-projected
    g1 = in_span if g1_reading == "projected" else V @ (V.T @ g)
    x = g_tilde - g1
    b_new = momentum * b + x
    o = -lr * b_new
    delta2 = o - V @ (V.T @ o)

    return w + delta1 + delta2, b_new


def fosi_step_adamw(w: np.ndarray, g: np.ndarray, V: np.ndarray, evals: np.ndarray, exp_avg: np.ndarray,
                    exp_avg_sq: np.ndarray, step_index: int, alpha: float, lr: float, beta1: float, beta2: float,
                    eps: float, weight_decay: float, sigma: float = 0.0, pi: Optional[np.ndarray] = None,
                    curv_mode: str = "signed") -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """The same update with AdamW as the base optimiser (the optimiser of the paper's experiments, Section IV).
    Returns (w_new, exp_avg_new, exp_avg_sq_new).

    Reading: the optimiser is handed x = g~ - g_1 and returns its whole descent vector
        o = -lr ( m_hat / (sqrt(v_hat) + eps) + weight_decay * w ),
    decoupled decay included, with the usual bias corrections for `step_index` (1-based); Eq. 12 / Eq. 14
    then re-project it: Delta_2 = o - V (V^T o).  With no columns in V this is textbook AdamW."""
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    a_hat = np.asarray(evals, dtype=np.float64)
    if pi is None:
        g_tilde, sig = g, 0.0
    else:
        g_tilde, sig = g + np.asarray(pi, dtype=np.float64), float(sigma)
    in_span = V @ (V.T @ g_tilde)                 # g_1 of Eq. 3 (with the dual variable added, Eq. 14)
    c = V.T @ in_span                             # Eq. 4 / Eq. 14 as printed
    denom = a_hat + sig if curv_mode == "signed" else np.abs(a_hat) + sig
    delta1 = -alpha * (V @ (c / denom))
    x = g_tilde - in_span
    m_new = beta1 * np.asarray(exp_avg, dtype=np.float64) + (1.0 - beta1) * x
    v_new = beta2 * np.asarray(exp_avg_sq, dtype=np.float64) + (1.0 - beta2) * x * x
    m_hat = m_new / (1.0 - beta1 ** step_index)
    v_hat = v_new / (1.0 - beta2 ** step_index)
    o = -lr * (m_hat / (np.sqrt(v_hat) + eps) + weight_decay * w)
    delta2 = o - V @ (V.T @ o)
    return w + delta1 + delta2, m_new, v_new
