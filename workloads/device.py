"""Large planted-spectrum workloads generated directly in GPU memory with torch
(the full-size configs would take minutes to draw and orthonormalise on the
host).  Same recipe as the host generator -- Gaussian block, two rounds of
Cholesky-QR in float64, fp32 storage -- but drawn from torch's seeded device
generator, so the values differ from the host generator's.  Input construction
only: none of the optimiser's arithmetic is here."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

from .generators import CONFIGS, ROOT_SEED, StepParams, padded_ld, planted_spectrum

CHUNK = 1 << 20


@dataclass
class PlantedDeviceWorkload:
    cfg_id: int
    n: int
    r: int
    m: int
    k: int
    l: int
    ld: int
    U: torch.Tensor        # flat fp32, column-major n x r with leading dimension ld
    lam: torch.Tensor      # r fp32
    shift: float
    v1: torch.Tensor       # n fp32
    w0: torch.Tensor       # n fp32
    g_std: float
    admm: bool
    steps: int
    params: StepParams

    def grad(self, t: int) -> torch.Tensor:
        gen = torch.Generator(device=self.U.device)
        gen.manual_seed(ROOT_SEED * 1000 + self.cfg_id * 100 + 10 + t)
        return torch.randn(self.n, generator=gen, device=self.U.device, dtype=torch.float32) * self.g_std


def _cholesky_qr_round(U: torch.Tensor, n: int, r: int, ld: int) -> None:
    """One in-place round: U <- U R^-1 with R^T R = U^T U, accumulated in float64 by row chunks."""
    M = U.view(r, ld)
    gram = torch.zeros(r, r, dtype=torch.float64, device=U.device)
    for lo in range(0, n, CHUNK):
        blk = M[:, lo:min(n, lo + CHUNK)].double()
        gram += blk @ blk.T
    R = torch.linalg.cholesky(gram.cpu()).T            # upper triangular, on the host in float64
    rinv_t = torch.linalg.inv(R).T.contiguous().to(U.device)
    for lo in range(0, n, CHUNK):
        hi = min(n, lo + CHUNK)
        M[:, lo:hi] = (rinv_t @ M[:, lo:hi].double()).float()


def planted_workload_device(cfg_id: int, n: int | None = None, device: str = "cuda:0") -> PlantedDeviceWorkload:
    c = CONFIGS[cfg_id]
    n = int(n if n is not None else c["n"])
    r = c["r"]
    ld = padded_ld(n)
    gen = torch.Generator(device=device)
    gen.manual_seed(ROOT_SEED * 1000 + cfg_id * 100)
    U = torch.empty(r * ld, dtype=torch.float32, device=device)
    M = U.view(r, ld)
    for j in range(r):                                 # column by column keeps the temporary small
        M[j].normal_(generator=gen)
    if ld > n:
        M[:, n:] = 0.0
    for _ in range(2):
        _cholesky_qr_round(U, n, r, ld)
    gen.manual_seed(ROOT_SEED * 1000 + cfg_id * 100 + 1)
    v1 = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
    gen.manual_seed(ROOT_SEED * 1000 + cfg_id * 100 + 3)
    w0 = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
    lam = torch.from_numpy(planted_spectrum(cfg_id)).to(device)
    return PlantedDeviceWorkload(
        cfg_id=cfg_id, n=n, r=r, m=c["m"], k=c["k"], l=c["l"], ld=ld, U=U, lam=lam,
        shift=float(np.float32(c["shift"])), v1=v1, w0=w0, g_std=c["g_std"], admm=c["admm"],
        steps=c["steps"], params=StepParams())
