"""Seeded generators for the five synthetic workloads.

Every tensor is drawn from a counter-based Philox stream keyed by
(ROOT_SEED, config id, tensor id, row-chunk id), so a tensor is the same no
matter in which order, or in how many pieces, it is generated.

The workloads stand in for the training runs the paper measures on (image
classifiers trained on public datasets); they keep only the scale of one
parameter block (n), the Lanczos length m and the number of requested
eigenpairs (k largest, l smallest).

Nothing here performs a step of the optimiser: the only linear algebra is the
orthonormalisation that turns a Gaussian matrix into the planted eigenvector
block U, which is part of *building the input*.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

ROOT_SEED = 250500982
CHUNK_ROWS = 1 << 20

# tensor ids
T_U0, T_V1, T_LAM, T_W0, T_X, T_W, T_LABELS = 0, 1, 2, 3, 4, 5, 6
T_GRAD0 = 10


@dataclass(frozen=True)
class StepParams:
    """Hyper-parameters of one update, held as fp32 values (the arithmetic type
    of the GPU path); both sides upcast these exact values."""
    alpha: np.float32 = np.float32(0.1)      # Newton scale
    lr: np.float32 = np.float32(0.01)        # learning rate of the base optimiser
    momentum: np.float32 = np.float32(0.9)   # heavy-ball coefficient
    sigma: np.float32 = np.float32(5e-4)     # ADMM penalty (only used with a dual variable)


# n, r, m, k, l, shift, gradient std, positive range, number of negatives, grid kind
CONFIGS = {
    1: dict(n=4096, r=32, m=40, k=10, l=0, shift=0.1, g_std=1.0,
            pos=(1e3, 1.0), n_neg=0, grid="geometric", admm=False, steps=1),
    2: dict(n=1 << 20, r=64, m=60, k=10, l=5, shift=0.01, g_std=0.1,
            pos=(1e4, 1e-1), n_neg=8, grid="geometric", admm=True, steps=10),
    3: dict(B=512, d=2048, C=1000, m=60, k=20, l=0),
    6: dict(B=8192, d=2048, C=1000, m=60, k=20, l=0, bf16=True),   # second softmax-GGN workload: larger batch, bf16 data
    4: dict(n=25_600_000, r=128, m=80, k=20, l=10, shift=0.01, g_std=float(np.sqrt(1e-3)),
            pos=(1e-2, 1e4), n_neg=16, grid="loguniform", admm=False, steps=1),
    5: dict(n=125_000_000, r=128, m=100, k=20, l=20, shift=1e-3, g_std=float(np.sqrt(1e-3)),
            pos=(1e-3, 1e5), n_neg=32, grid="loguniform", admm=True, steps=10),
}
NEG_RANGE = (5.0, 0.5)   # magnitudes of the planted negative eigenvalues


def philox(cfg_id: int, tensor_id: int, chunk_id: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence([ROOT_SEED, int(cfg_id), int(tensor_id), int(chunk_id)])
    return np.random.Generator(np.random.Philox(ss))


def padded_ld(n: int, multiple: int = 64) -> int:
    """Leading dimension for a column-major device matrix with n rows: the next
    multiple of `multiple` floats, nudged off large powers of two so that the
    columns of a tall matrix do not all start on the same DRAM channel."""
    ld = (n + multiple - 1) // multiple * multiple
    if ld % 4096 == 0:
        ld += multiple
    return ld


def normal_vector(cfg_id: int, tensor_id: int, n: int, std: float = 1.0) -> np.ndarray:
    out = np.empty(n, dtype=np.float32)
    for c, lo in enumerate(range(0, n, CHUNK_ROWS)):
        hi = min(n, lo + CHUNK_ROWS)
        out[lo:hi] = philox(cfg_id, tensor_id, c).standard_normal(hi - lo, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def normal_matrix(cfg_id: int, tensor_id: int, n: int, r: int) -> np.ndarray:
    """n x r fp32, Fortran (column-major) order."""
    out = np.empty((n, r), dtype=np.float32, order="F")
    for c, lo in enumerate(range(0, n, CHUNK_ROWS)):
        hi = min(n, lo + CHUNK_ROWS)
        out[lo:hi, :] = philox(cfg_id, tensor_id, c).standard_normal((hi - lo, r), dtype=np.float32)
    return out


def orthonormal_columns(A: np.ndarray) -> np.ndarray:
    """Orthonormal basis of the column space of the tall matrix A, as fp32 in
    column-major order.  Small inputs: Householder QR in fp64.  Large inputs:
    two rounds of Cholesky-QR in fp64, chunked over rows (a Gaussian n x r
    matrix with n >> r is very well conditioned, so two rounds reach fp64
    orthogonality)."""
    n, r = A.shape
    if n <= (1 << 16):
        q, rr = np.linalg.qr(A.astype(np.float64))
        q *= np.sign(np.diag(rr))[None, :]
        return np.asfortranarray(q.astype(np.float32))
    cur = A
    for _ in range(2):
        gram = np.zeros((r, r))
        for lo in range(0, n, CHUNK_ROWS):
            blk = np.asarray(cur[lo:lo + CHUNK_ROWS], dtype=np.float64)
            gram += blk.T @ blk
        rinv = np.linalg.inv(np.linalg.cholesky(gram).T)
        nxt = np.empty((n, r), dtype=np.float64, order="F")
        for lo in range(0, n, CHUNK_ROWS):
            nxt[lo:lo + CHUNK_ROWS] = np.asarray(cur[lo:lo + CHUNK_ROWS], dtype=np.float64) @ rinv
        cur = nxt
    return np.asfortranarray(cur.astype(np.float32))


def planted_spectrum(cfg_id: int) -> np.ndarray:
    """The r planted eigenvalues (before the shift), fp32: positives first
    (descending for the geometric grids), then the negatives."""
    c = CONFIGS[cfg_id]
    r, n_neg = c["r"], c["n_neg"]
    hi, lo = max(c["pos"]), min(c["pos"])
    if c["grid"] == "geometric":
        pos = np.geomspace(hi, lo, r - n_neg)
        neg = -np.geomspace(NEG_RANGE[0], NEG_RANGE[1], n_neg) if n_neg else np.zeros(0)
    else:
        g = philox(cfg_id, T_LAM)
        pos = np.exp(g.uniform(np.log(lo), np.log(hi), r - n_neg))
        neg = -np.exp(g.uniform(np.log(NEG_RANGE[1]), np.log(NEG_RANGE[0]), n_neg))
    return np.concatenate([pos, neg]).astype(np.float32)


@dataclass
class PlantedWorkload:
    cfg_id: int
    n: int
    r: int
    m: int
    k: int
    l: int
    U: np.ndarray            # n x r fp32 column-major, orthonormal columns
    lam: np.ndarray          # r fp32
    shift: np.float32
    v1: np.ndarray           # n fp32, unnormalised N(0,1) start vector
    w0: np.ndarray           # n fp32 initial parameters
    g_std: float
    admm: bool
    steps: int
    params: StepParams = field(default_factory=StepParams)

    def grad(self, t: int) -> np.ndarray:
        return gradient(self.cfg_id, t, self.n, self.g_std)


def gradient(cfg_id: int, t: int, n: int, std: float) -> np.ndarray:
    return normal_vector(cfg_id, T_GRAD0 + t, n, std)


def planted_workload(cfg_id: int, n: Optional[int] = None) -> PlantedWorkload:
    """Host-side planted-spectrum workload H = U diag(lam) U^T + shift I.
    `n` overrides the row count (reduced-size variants of the large configs
    keep r, m, k, l and the spectrum)."""
    c = CONFIGS[cfg_id]
    n = int(n if n is not None else c["n"])
    r = c["r"]
    U = orthonormal_columns(normal_matrix(cfg_id, T_U0, n, r))
    return PlantedWorkload(
        cfg_id=cfg_id, n=n, r=r, m=c["m"], k=c["k"], l=c["l"], U=U,
        lam=planted_spectrum(cfg_id), shift=np.float32(c["shift"]),
        v1=normal_vector(cfg_id, T_V1, n), w0=normal_vector(cfg_id, T_W0, n),
        g_std=c["g_std"], admm=c["admm"], steps=c["steps"])


@dataclass
class GgnWorkload:
    B: int
    d: int
    C: int
    m: int
    k: int
    l: int
    X: np.ndarray        # B x d fp32 row-major
    W: np.ndarray        # d x C fp32 row-major
    labels: np.ndarray   # B int64 (not used by the curvature; generated for completeness)
    v1: np.ndarray       # d*C fp32

    @property
    def n(self) -> int:
        return self.d * self.C


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array rounded to the nearest bf16 value (ties to even), returned as fp32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(a))


def ggn_workload(B: Optional[int] = None, d: Optional[int] = None, C: Optional[int] = None,
                 m: Optional[int] = None, k: Optional[int] = None, cfg_id: int = 3, bf16: Optional[bool] = None) -> GgnWorkload:
    """Softmax-GGN workload.  cfg_id 3: the small-batch fp32 one; cfg_id 6: the larger batch whose data
    matrix is stored in bf16 (X is then rounded to bf16 values, still returned as fp32)."""
    c = CONFIGS[cfg_id]
    B, d, C = int(B or c["B"]), int(d or c["d"]), int(C or c["C"])
    X = (philox(3, T_X).standard_normal((B, d), dtype=np.float32) * np.float32(1.0 / np.sqrt(d)))
    if c.get("bf16", False) if bf16 is None else bf16:
        X = round_to_bf16(X)
    W = philox(3, T_W).standard_normal((d, C), dtype=np.float32)
    labels = philox(3, T_LABELS).integers(0, C, B)
    v1 = philox(3, T_V1).standard_normal(d * C, dtype=np.float32)
    return GgnWorkload(B=B, d=d, C=C, m=int(m or c["m"]), k=int(k or c["k"]), l=c["l"],
                       X=np.ascontiguousarray(X), W=np.ascontiguousarray(W), labels=labels, v1=v1)
