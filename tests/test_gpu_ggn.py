"""GPU parity of the softmax-GGN operator (the MFMA path) and of the curvature
step built on it, against the CPU oracle.

Tolerance of one operator application: the two GEMMs accumulate in fp32 on the
matrix cores over K = d and K = B terms; with random-sign rounding the relative
error grows like sqrt(K) * 2^-24 (about 3e-6 at d = 2048), so 2e-5 relative L2
is required.  Ritz values / subspaces keep the path-wide bars (1e-4, 1e-3 rad).
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from tests.helpers import rel_l2, sin_principal_angles

pytestmark = pytest.mark.gpu
GGN_RTOL = 2e-5


@pytest.fixture(scope="module")
def fo():
    import paper_2505_00982_amd as fo
    return fo


@pytest.fixture(scope="module")
def ctx(fo):
    c = fo.Context(0)
    yield c
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


# (70, 200, 132), (130, 260, 100), (4, 4, 4): every extent a multiple of 4, so both products take the kernel for
# aligned shapes with ragged tiles in M, N and K; the odd shapes take the generic kernel
# C = 1500, 2500: the softmax-Jacobian row kept in 8 registers per thread / too long for registers (two-pass kernel);
# (96, 64, 36), (32, 32, 4): both contraction lengths multiples of 32 (whole K-steps: the variant with constant address
# increments), ragged in M and N
# (8192, 64, 1000), (64, 8192, 1000): 2048 output tiles of 64 x 64 in the first / the second product, which then takes
# the 128-row tile; (8192, 72, 1000): the same with a contraction length that is not a whole number of K-steps
@pytest.mark.parametrize("B,d,C", [(16, 8, 5), (1, 1, 1), (70, 200, 132), (130, 260, 100), (4, 4, 4), (100, 301, 130),
                                   (65, 17, 64), (9, 12, 1500), (9, 12, 2500), (96, 64, 36), (32, 32, 4), (512, 2048, 1000),
                                   (8192, 64, 1000), (64, 8192, 1000), (8192, 72, 1000)])
def test_ggn_operator_matches_oracle(fo, ctx, B, d, C):
    g = wl.ggn_workload(B=B, d=d, C=C)
    op = ctx.hvp_softmax_ggn(dev(g.X), dev(g.W))
    for seed in (60, 61):
        v = wl.normal_vector(3, seed, g.n)
        out = torch.zeros(g.n, device="cuda")
        op.apply(dev(v), out)
        ctx.synchronize()
        ref = oracle.hvp_softmax_ggn(g.X, g.W, v)
        assert rel_l2(out.cpu().numpy(), ref) <= GGN_RTOL
    op.close()


@pytest.mark.parametrize("B,d,C", [(96, 64, 36), (512, 2048, 1000), (8192, 64, 1000), (64, 8192, 1000)])
def test_ggn_operator_register_staged_kernels(fo, B, d, C, monkeypatch):
    """FOSI_GGN_DIRECT=0 at context creation sends the shapes that normally load their tiles straight into LDS
    through the register-staged kernels (the path of contraction lengths that are not whole K-steps)."""
    monkeypatch.setenv("FOSI_GGN_DIRECT", "0")
    c = fo.Context(0)
    try:
        g = wl.ggn_workload(B=B, d=d, C=C)
        op = c.hvp_softmax_ggn(dev(g.X), dev(g.W))
        v = wl.normal_vector(3, 63, g.n)
        out = torch.zeros(g.n, device="cuda")
        op.apply(dev(v), out)
        c.synchronize()
        assert rel_l2(out.cpu().numpy(), oracle.hvp_softmax_ggn(g.X, g.W, v)) <= GGN_RTOL
        op.close()
    finally:
        c.close()


def test_ggn_operator_properties(fo, ctx):
    g = wl.ggn_workload(B=64, d=96, C=40)
    op = ctx.hvp_softmax_ggn(dev(g.X), dev(g.W))
    u, v = wl.normal_vector(3, 70, g.n), wl.normal_vector(3, 71, g.n)
    hu, hv = torch.zeros(g.n, device="cuda"), torch.zeros(g.n, device="cuda")
    op.apply(dev(u), hu)
    op.apply(dev(v), hv)
    ctx.synchronize()
    hu, hv = hu.cpu().numpy().astype(np.float64), hv.cpu().numpy().astype(np.float64)
    assert abs(u @ hv - v @ hu) <= 1e-5 * (np.linalg.norm(u) * np.linalg.norm(hv))     # symmetry
    assert v @ hv >= 0                                                                   # positive semi-definite
    shift_dir = np.outer(wl.normal_vector(3, 72, g.d), np.ones(g.C)).reshape(-1).astype(np.float32)
    hs = torch.zeros(g.n, device="cuda")
    op.apply(dev(shift_dir), hs)
    ctx.synchronize()
    assert np.linalg.norm(hs.cpu().numpy()) <= 1e-5 * np.linalg.norm(hv)                 # class-shift null space
    op.close()


def _ggn_curvature(fo, ctx, g, m, k):
    op = ctx.hvp_softmax_ggn(dev(g.X), dev(g.W))
    ld = wl.padded_ld(g.n)
    Q = fo.ColMajor(g.n, m + 1, ld)
    Q.col(0).copy_(dev(g.v1))
    alpha, beta, m_eff = fo.fosi_lanczos(ctx, op, Q, m)
    V = fo.ColMajor(g.n, k, ld)
    evals, resid = fo.fosi_ritz(ctx, Q, m_eff, alpha, beta, k, 0, V)
    ctx.synchronize()
    res = oracle.lanczos(lambda v: oracle.hvp_softmax_ggn(g.X, g.W, v), g.v1, m)
    rz = oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, k, 0)
    op.close()
    return dict(alpha=alpha, beta=beta, m_eff=m_eff, evals=evals, resid=resid, V=V, Q=Q), res, rz


def test_ggn_curvature_small(fo, ctx):
    g = wl.ggn_workload(B=64, d=96, C=40, m=30, k=6)
    gp, res, rz = _ggn_curvature(fo, ctx, g, 30, 6)
    assert gp["m_eff"] == res.m_eff == 30
    assert np.max(np.abs(gp["evals"] - rz.evals) / np.abs(rz.evals)) <= 1e-4
    assert sin_principal_angles(rz.V, gp["V"].to_numpy()).max() < 1e-3
    Q = gp["Q"].to_numpy(30).astype(np.float64)
    assert np.abs(Q.T @ Q - np.eye(30)).max() < 1e-5


def test_ggn_curvature_reference_size(fo, ctx):
    """W of shape 2048 x 1000, batch 512, m = 60, k = 20 (the third workload) at full size."""
    g = wl.ggn_workload()
    gp, res, rz = _ggn_curvature(fo, ctx, g, g.m, g.k)
    assert gp["m_eff"] == res.m_eff == g.m
    rel = np.abs(gp["evals"] - rz.evals) / np.abs(rz.evals)
    assert rel.max() <= 1e-4, rel
    # Ritz vectors: compare as a subspace those pairs the oracle itself has resolved (residual small against the
    # value); all k of them are then checked one by one below
    conv = rz.resid <= 1e-3 * np.abs(rz.evals)
    assert conv.sum() >= 5
    idx = np.arange(g.k)[conv]
    # a converged block is only a well-defined subspace if it is contiguous from the top
    top = idx[: (np.diff(idx, prepend=-1) == 1).cumprod().sum()]
    Vg = gp["V"].to_numpy().astype(np.float64)
    assert sin_principal_angles(rz.V[:, top], Vg[:, top]).max() < 1e-3
    # Every one of the k vectors, resolved or not: it is a unit vector orthogonal to the others, its residual
    # under the oracle's float64 operator is the one the oracle's own pair has (for a Ritz pair of a Krylov space
    # ||H v - theta v|| = |beta_m s_mi| exactly, so a vector that is not the Ritz vector of its value shows here),
    # and the residual estimate the library returns is the same number.
    assert np.abs(Vg.T @ Vg - np.eye(g.k)).max() <= 1e-5
    scale = np.abs(rz.evals).max()
    true_resid = np.array([np.linalg.norm(oracle.hvp_softmax_ggn(g.X, g.W, Vg[:, i]) - gp["evals"][i] * Vg[:, i])
                           for i in range(g.k)])
    assert np.abs(true_resid - rz.resid).max() <= 1e-4 * scale, (true_resid, rz.resid)
    assert np.abs(np.asarray(gp["resid"]) - rz.resid).max() <= 1e-4 * scale
    # and inside the span of the oracle's own Krylov basis each vector has the oracle's coefficients (this is a
    # comparison of all k columns, one by one, up to sign; what it leaves out is the part outside that span,
    # bounded by the orthonormality and residual checks above)
    coef_g = res.Q[:, : g.m].T @ Vg                                    # m x k
    coef_o = res.Q[:, : g.m].T @ rz.V
    sign = np.sign(np.sum(coef_g * coef_o, axis=0))
    per_pair = np.linalg.norm(coef_g * sign - coef_o, axis=0)
    gap = np.array([np.sort(np.abs(rz.all_evals - e))[1] for e in rz.evals])     # distance to the nearest other Ritz value
    print("cfg3 per-pair coefficient deviation", np.array2string(per_pair, precision=2), "resid/gap", np.array2string(rz.resid / gap, precision=2))
    assert (per_pair < 1e-3).all(), per_pair
    whole = np.array([np.linalg.norm(Vg[:, i] - (rz.V[:, i] @ Vg[:, i]) * rz.V[:, i]) for i in range(g.k)])
    print("cfg3 per-pair sine of the angle between the library's and the oracle's vector", np.array2string(whole, precision=2))
    assert (whole < 1e-3).all(), whole


# ------------------------------------------------------------------ bf16 data matrix, split-operand matrix-core path
def dev_bf16(a):
    """bf16 tensor holding exactly the (already bf16-representable) fp32 values of `a`."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(torch.bfloat16)
    assert torch.equal(t.float().cpu(), torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)))
    return t.contiguous()


# shapes: single partial tile; unaligned row length (scalar staging path); several tiles with ragged edges in
# every dimension; d, B multiples of the K step; a shape that splits both products along K
@pytest.mark.parametrize("B,d,C", [(16, 8, 5), (1, 1, 1), (70, 200, 132), (100, 301, 130), (257, 96, 300), (640, 512, 250)])
def test_ggn_bf16_operator_matches_oracle(fo, ctx, B, d, C):
    g = wl.ggn_workload(B=B, d=d, C=C, bf16=True)
    op = ctx.hvp_softmax_ggn_bf16(dev_bf16(g.X), dev(g.W))
    for seed in (60, 61):
        v = wl.normal_vector(3, seed, g.n)
        out = torch.zeros(g.n, device="cuda")
        op.apply(dev(v), out)
        ctx.synchronize()
        ref = oracle.hvp_softmax_ggn(g.X, g.W, v)      # the oracle sees the same bf16-exact X, in fp64
        assert rel_l2(out.cpu().numpy(), ref) <= GGN_RTOL
    op.close()


def test_ggn_bf16_curvature(fo, ctx):
    g = wl.ggn_workload(B=300, d=160, C=50, m=30, k=6, bf16=True)
    op = ctx.hvp_softmax_ggn_bf16(dev_bf16(g.X), dev(g.W))
    ld = wl.padded_ld(g.n)
    Q = fo.ColMajor(g.n, g.m + 1, ld)
    Q.col(0).copy_(dev(g.v1))
    alpha, beta, m_eff = fo.fosi_lanczos(ctx, op, Q, g.m)
    V = fo.ColMajor(g.n, g.k, ld)
    evals, _ = fo.fosi_ritz(ctx, Q, m_eff, alpha, beta, g.k, 0, V)
    ctx.synchronize()
    res = oracle.lanczos(lambda v: oracle.hvp_softmax_ggn(g.X, g.W, v), g.v1, g.m)
    rz = oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, g.k, 0)
    assert m_eff == res.m_eff == g.m
    assert np.max(np.abs(evals - rz.evals) / np.abs(rz.evals)) <= 1e-4
    conv = rz.resid <= 1e-3 * np.abs(rz.evals)
    idx = np.arange(g.k)[conv]
    top = idx[: (np.diff(idx, prepend=-1) == 1).cumprod().sum()]
    assert len(top) >= 2
    assert sin_principal_angles(rz.V[:, top], V.to_numpy()[:, top]).max() < 1e-3
    op.close()


def test_ggn_bf16_larger_batch_sampled(fo, ctx):
    """The second softmax-GGN workload at full size (batch 8192, W 2048 x 1000): the whole result against
    the fp64 oracle (two float64 GEMMs of 33 GFLOP on the host)."""
    g = wl.ggn_workload(cfg_id=6)
    op = ctx.hvp_softmax_ggn_bf16(dev_bf16(g.X), dev(g.W))
    v = wl.normal_vector(3, 62, g.n)
    out = torch.zeros(g.n, device="cuda")
    op.apply(dev(v), out)
    ctx.synchronize()
    ref = oracle.hvp_softmax_ggn(g.X, g.W, v)
    assert rel_l2(out.cpu().numpy(), ref) <= GGN_RTOL
    op.close()
