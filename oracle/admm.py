"""Outer ADMM-like bookkeeping of Algorithm 3 (and Eq. 11), float64.  Test
infrastructure only.

At the start of outer iteration k the anchor is w = w_a + pi / sigma and the
working copy w_a restarts from it; after the inner updates the multiplier
becomes pi + sigma (w_a - w).  (Eq. 15 starts w_a from the previous anchor;
Algorithm 3, which is followed here, starts it from the new one.)
"""
from __future__ import annotations

from typing import Tuple

import numpy as np


def admm_begin(w_a: np.ndarray, pi: np.ndarray, sigma: float) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (w_anchor, w_a_restart)."""
    w = np.asarray(w_a, dtype=np.float64) + np.asarray(pi, dtype=np.float64) / float(sigma)
    return w, w.copy()


def admm_end(w_anchor: np.ndarray, w_a: np.ndarray, pi: np.ndarray, sigma: float) -> np.ndarray:
    """Returns the new multiplier."""
    return np.asarray(pi, dtype=np.float64) + float(sigma) * (
        np.asarray(w_a, dtype=np.float64) - np.asarray(w_anchor, dtype=np.float64))
