"""CPU oracle for the curvature step and the hybrid-order update (TEST INFRASTRUCTURE).

A plain, slow, float64 numpy transcription of what the hot path computes:
Lanczos with full Gram-Schmidt (Algorithm 1), Ritz extraction (Eq. 8 and the
paragraph after it), the two-subspace update (Eq. 4 and Eq. 12; Eq. 14 with the
dual variable) and the outer multiplier update (Eq. 11, Algorithm 3).

This package exists only to be compared against.  It shares no code with the
HIP library, never imports it, and must not be imported by the product path:
only tests, the smoke check and the `cpu_baseline` leg of the benchmark call it.

Parity status: every function here is pinned by CPU tests to facts it does not
compute itself (planted spectra, dense eigendecomposition, Householder
tridiagonalisation of the reduced problem, a library SGD, autograd Hessian
products, closed forms).  No function is "parity unpinned".
"""
from .hvp import hvp_planted, hvp_diag, hvp_softmax_ggn, softmax_rows  # noqa: F401
from .lanczos import lanczos, LanczosResult  # noqa: F401
from .ritz import ritz, RitzResult  # noqa: F401
from .step import fosi_step, fosi_step_adamw  # noqa: F401
from .admm import admm_begin, admm_end  # noqa: F401
