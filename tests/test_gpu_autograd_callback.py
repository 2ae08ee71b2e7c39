"""The operator the paper actually uses: H v from a network by double back-propagation (the paper cites
Pearlmutter's algorithm in the paragraph introducing Algorithm 1), fed to the HIP Lanczos through
`hvp_callback_create`.  The callback runs torch autograd on the GPU in fp32; the oracle runs the same
network in float64 on the CPU."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from tests.helpers import sin_principal_angles

pytestmark = pytest.mark.gpu

SIZES = [(12, 24), (24, 16), (16, 3)]   # a small tanh MLP: 12 -> 24 -> 16 -> 3
N_PARAMS = sum(i * o + o for i, o in SIZES)


def _unflatten(flat):
    out, off = [], 0
    for i, o in SIZES:
        W = flat[off: off + i * o].reshape(i, o)
        off += i * o
        b = flat[off: off + o]
        off += o
        out.append((W, b))
    return out


def _loss(flat, X, Y):
    h = X
    layers = _unflatten(flat)
    for idx, (W, b) in enumerate(layers):
        h = h @ W + b
        if idx + 1 < len(layers):
            h = torch.tanh(h)
    return torch.mean((h - Y) ** 2)


def _hvp(flat, X, Y, v):
    flat = flat.detach().requires_grad_(True)
    g, = torch.autograd.grad(_loss(flat, X, Y), flat, create_graph=True)
    hv, = torch.autograd.grad(g @ v, flat)
    return hv


def test_lanczos_on_autograd_hessian():
    import paper_2505_00982_amd as fo
    rng = np.random.default_rng(21)
    w0 = (0.5 * rng.standard_normal(N_PARAMS)).astype(np.float32)
    X = rng.standard_normal((64, SIZES[0][0])).astype(np.float32)
    Y = rng.standard_normal((64, SIZES[-1][1])).astype(np.float32)
    v1 = wl.normal_vector(1, 95, N_PARAMS)
    m, k, l = 40, 5, 3

    ctx = fo.Context(0)
    wd, Xd, Yd = (torch.from_numpy(a).cuda() for a in (w0, X, Y))
    Q = fo.ColMajor(N_PARAMS, m + 1)
    Q.col(0).copy_(torch.from_numpy(v1).cuda())

    def cb(v_ptr, hv_ptr, stream):
        jv = (v_ptr - Q.ptr) // (4 * Q.ld)
        jh = (hv_ptr - Q.ptr) // (4 * Q.ld)
        Q.col(jh).copy_(_hvp(wd, Xd, Yd, Q.col(jv)))
        return 0

    op = ctx.hvp_callback(N_PARAMS, cb)
    alpha, beta, m_eff = fo.fosi_lanczos(ctx, op, Q, m)
    V = fo.ColMajor(N_PARAMS, k + l)
    evals, _ = fo.fosi_ritz(ctx, Q, m_eff, alpha, beta, k, l, V)
    ctx.synchronize()

    w64, X64, Y64 = (torch.from_numpy(a.astype(np.float64)) for a in (w0, X, Y))
    op_ref = lambda v: _hvp(w64, X64, Y64, torch.from_numpy(np.asarray(v, dtype=np.float64))).numpy()
    res = oracle.lanczos(op_ref, v1, m)
    rz = oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, k, l)
    assert m_eff == res.m_eff == m
    scale = np.abs(rz.all_evals).max()
    # the fp32 autograd operator itself carries ~1e-6 relative error; compare the top values tightly and the
    # (small, possibly unresolved) bottom ones on the scale of the operator
    assert np.max(np.abs(evals[:k] - rz.evals[:k]) / np.abs(rz.evals[:k])) <= 1e-4
    assert np.max(np.abs(evals[k:] - rz.evals[k:])) <= 1e-4 * scale
    conv = rz.resid[:k] <= 1e-3 * np.abs(rz.evals[:k])
    top = np.arange(k)[: int(np.cumprod(conv).sum())]
    assert len(top) >= 2
    assert sin_principal_angles(rz.V[:, top], V.to_numpy()[:, top]).max() < 1e-3
    Qh = Q.to_numpy(m).astype(np.float64)
    assert np.abs(Qh.T @ Qh - np.eye(m)).max() < 1e-5
    op.close()
    ctx.close()
