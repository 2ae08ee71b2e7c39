"""GPU parity at the benchmark's sizes.

Workload 2 (n = 2^20) is small enough for the complete CPU oracle.  Workload 4
(n = 25.6 M, the configuration bench.py times) is too large for it, so the HIP
path is checked there through (a) the tridiagonal obtained by an independent
route (Householder reduction of the operator restricted to span([U, v1]), which
needs only a small Gram matrix, accumulated in float64 by library matmuls),
(b) invariants evaluated with library float64 operations, and (c) sampled rows
of the Ritz vectors and of the update, which the oracle's formulas give one by
one."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from oracle.lanczos import tridiagonal
from tests.helpers import (reduced_ritz_coefficients, reduced_tridiagonal_from_gram, rel_l2,
                           sin_principal_angles)

pytestmark = pytest.mark.gpu


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


def test_workload2_full_size_against_complete_oracle(fo, ctx):
    w = wl.planted_workload(2)
    ld = wl.padded_ld(w.n)
    U = fo.ColMajor.from_numpy(w.U, ld)
    op = ctx.hvp_planted(U, dev(w.lam), float(w.shift))
    Q = fo.ColMajor(w.n, w.m + 1, ld)
    Q.col(0).copy_(dev(w.v1))
    alpha, beta, m_eff = fo.fosi_lanczos(ctx, op, Q, w.m)
    r_v = w.k + w.l
    V = fo.ColMajor(w.n, r_v, ld)
    evals, resid = fo.fosi_ritz(ctx, Q, m_eff, alpha, beta, w.k, w.l, V)
    ctx.synchronize()

    res = oracle.lanczos(lambda v: oracle.hvp_planted(w.U, w.lam, float(w.shift), v), w.v1, w.m)
    rz = oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, w.k, w.l)
    assert m_eff == res.m_eff == w.m
    scale = np.abs(w.lam).max()
    assert np.max(np.abs(alpha - res.alpha)) < 1e-5 * scale and np.max(np.abs(beta - res.beta)) < 1e-5 * scale
    assert np.max(np.abs(evals - rz.evals) / np.abs(rz.evals)) <= 1e-4
    Vg = V.to_numpy().astype(np.float64)
    assert sin_principal_angles(rz.V[:, : w.k], Vg[:, : w.k]).max() < 1e-3
    assert sin_principal_angles(rz.V[:, w.k:], Vg[:, w.k:]).max() < 1e-3

    # one outer iteration of Algorithm 3: anchor, ten updates with fresh gradients, multiplier update
    p = w.params
    sig = float(p.sigma)
    sp = fo.StepParams(float(p.alpha), float(p.lr), float(p.momentum), sig, 0)
    pi0 = (1e-3 * wl.normal_vector(2, 40, w.n)).astype(np.float32)
    wa, pi = dev(w.w0), dev(pi0)
    mom, anchor = torch.zeros(w.n, device="cuda"), torch.zeros(w.n, device="cuda")
    fo.fosi_admm_begin(ctx, sig, pi, anchor, wa)
    for t in range(w.steps):
        fo.fosi_step(ctx, V, r_v, evals, dev(w.grad(t)), pi, mom, wa, sp)
    fo.fosi_admm_end(ctx, sig, anchor, wa, pi)
    ctx.synchronize()
    _, wa_ref = oracle.admm_begin(w.w0, pi0, sig)
    b_ref = np.zeros(w.n)
    for t in range(w.steps):
        wa_ref, b_ref = oracle.fosi_step(wa_ref, w.grad(t), Vg, evals, b_ref, float(p.alpha), float(p.lr),
                                         float(p.momentum), sig, pi=pi0)
    assert rel_l2(wa.cpu().numpy(), wa_ref) <= 1e-5
    assert rel_l2(mom.cpu().numpy(), b_ref) <= 1e-5
    pi_ref = oracle.admm_end(anchor.cpu().numpy(), wa.cpu().numpy(), pi0, sig)
    assert rel_l2(pi.cpu().numpy(), pi_ref) <= 1e-6
    op.close()


def _gram_f64(M: torch.Tensor, n: int, extra: torch.Tensor, chunk: int = 1 << 20) -> np.ndarray:
    """Gram matrix of [rows of M transposed | extra] in float64, by row chunks (library matmul)."""
    c = M.shape[0]
    G = torch.zeros(c + 1, c + 1, dtype=torch.float64, device=M.device)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        blk = torch.cat([M[:, lo:hi].double(), extra[lo:hi].double()[None, :]], dim=0)
        G += blk @ blk.T
    return G.cpu().numpy()


def _full_size_planted(fo, ctx, cfg_id):
    from workloads.device import planted_workload_device
    w = planted_workload_device(cfg_id)
    n, m, r = w.n, w.m, w.r
    U = fo.ColMajor(n, r, w.ld, buf=w.U)
    op = ctx.hvp_planted(U, w.lam, w.shift)
    Q = fo.ColMajor(n, m + 1, w.ld)
    Q.col(0).copy_(w.v1)
    alpha, beta, m_eff = fo.fosi_lanczos(ctx, op, Q, m)
    r_v = w.k + w.l
    V = fo.ColMajor(n, r_v, w.ld)
    evals, resid = fo.fosi_ritz(ctx, Q, m_eff, alpha, beta, w.k, w.l, V)
    ctx.synchronize()
    assert m_eff == m
    lam = w.lam.cpu().numpy().astype(np.float64)
    scale = np.abs(lam).max()

    # (a) tridiagonal by the independent route
    G = _gram_f64(w.U.view(r, w.ld), n, w.v1)
    a_ref, b_ref = reduced_tridiagonal_from_gram(G, lam, w.shift)
    assert np.max(np.abs(alpha[:40] - a_ref[:40])) < 1e-5 * scale
    assert np.max(np.abs(beta[:40] - b_ref[:40])) < 1e-5 * scale
    # Ritz values and the reference Ritz vectors V_ref = [U, v1] C from the same independent route.  Pairs the
    # fp64 reference has resolved (residual estimate <= 1e-2 |theta|) must agree to 1e-4 relative.  For the
    # others the bar follows from the arithmetic: storing the basis in fp32 perturbs the operator by about
    # u32 ||H|| per step, and an unresolved Ritz value can move by that much (4 u32 ||H|| allowed).
    u32 = 2.0 ** -24
    ev_ref, Cmat, resid_ref, all_ref = reduced_ritz_coefficients(G, lam, w.shift, m, w.k, w.l)
    resolved_all = resid_ref <= 1e-2 * np.abs(ev_ref)
    err = np.abs(evals - ev_ref)
    print(f"[workload {cfg_id}] Ritz value relative errors {np.array2string(err / np.abs(ev_ref), precision=1)}; "
          f"resolved by the reference: {resolved_all.sum()} of {r_v}")
    assert resolved_all.sum() >= w.k
    assert np.max(err[resolved_all] / np.abs(ev_ref[resolved_all])) <= 1e-4
    assert np.max(err) <= max(1e-4 * np.abs(ev_ref).min(), 4 * u32 * scale)
    Vm_ = V.buf[: r_v * w.ld].view(r_v, w.ld)
    Um_ = w.U.view(r, w.ld)
    cross = torch.zeros(r_v, r + 1, dtype=torch.float64, device="cuda")
    for lo in range(0, n, 1 << 20):
        hi = min(n, lo + (1 << 20))
        basis = torch.cat([Um_[:, lo:hi].double(), w.v1[lo:hi].double()[None, :]], dim=0)
        cross += Vm_[:, lo:hi].double() @ basis.T
    overlap = cross.cpu().numpy() @ Cmat                       # V_gpu^T V_ref, r_v x r_v
    for name, blk, outside in (("top", slice(0, w.k), all_ref[m - 1 - w.k]), ("bottom", slice(w.k, r_v), all_ref[w.l])):
        sv = np.linalg.svd(overlap[blk, blk], compute_uv=False)
        sines = np.sqrt(np.maximum(0.0, 1.0 - np.minimum(sv, 1.0) ** 2))
        # per pair: how far the GPU's Ritz vector leaves the reference block
        leave = np.sqrt(np.maximum(0.0, 1.0 - np.sum(overlap[blk, blk] ** 2, axis=1)))
        gap = np.min(np.abs(ev_ref[blk] - outside))
        print(f"[workload {cfg_id}] {name} block: max sin(angle) {sines.max():.2e}; per pair {np.array2string(leave, precision=1)}; "
              f"reference residuals {np.array2string(resid_ref[blk], precision=1)}; gap to the next Ritz value {gap:.3f}")
        resolved = resid_ref[blk] <= 1e-2 * np.abs(ev_ref[blk])
        # pairs the fp64 reference has resolved: the 1e-3 rad bar
        assert leave[resolved].max() < 1e-3
        # the whole block, unresolved pairs included: fp32 storage of the basis perturbs the operator by
        # ~u32 ||H|| per step, and a Ritz vector moves by about that over the gap to the next Ritz value
        assert sines.max() < max(1e-3, 16 * u32 * scale / gap)

    # (b) invariants with library float64 operations
    Qm = Q.buf[: (m + 1) * w.ld].view(m + 1, w.ld)
    Gq = torch.zeros(m, m, dtype=torch.float64, device="cuda")
    for lo in range(0, n, 1 << 20):
        blk = Qm[:m, lo:min(n, lo + (1 << 20))].double()
        Gq += blk @ blk.T
    assert (Gq - torch.eye(m, dtype=torch.float64, device="cuda")).abs().max().item() < 1e-5
    Vm = V.buf[: r_v * w.ld].view(r_v, w.ld)
    Gv = torch.zeros(r_v, r_v, dtype=torch.float64, device="cuda")
    for lo in range(0, n, 1 << 20):
        blk = Vm[:, lo:min(n, lo + (1 << 20))].double()
        Gv += blk @ blk.T
    assert (Gv - torch.eye(r_v, dtype=torch.float64, device="cuda")).abs().max().item() < 1e-5

    # (c) sampled rows of the Ritz vectors: V[rows] = Q[rows, :m] S with S from LAPACK on the GPU's own T
    rows = torch.from_numpy(np.random.default_rng(7).choice(n, 4096, replace=False)).cuda()
    uT, ST = np.linalg.eigh(tridiagonal(alpha, beta, m))
    sel = np.concatenate([np.arange(m - 1, m - 1 - w.k, -1), np.arange(w.l)])
    Qs = Qm[:m][:, rows].double().cpu().numpy().T           # 4096 x m
    Vs = Vm[:, rows].double().cpu().numpy().T               # 4096 x r_v
    ref = Qs @ ST[:, sel]
    sign = np.sign(np.sum(ref * Vs, axis=0))
    assert np.max(np.abs(ref * sign - Vs)) <= 2e-6 * np.sqrt(m) * np.abs(Qs).max()

    # (c) sampled rows of one update; the two small coefficient vectors come from library float64 products
    p = w.params
    sp = fo.StepParams(float(p.alpha), float(p.lr), float(p.momentum), float(p.sigma), 0)
    g = w.grad(0)
    wa, mom = w.w0.clone(), torch.zeros(n, device="cuda")
    c = torch.zeros(r_v, dtype=torch.float64, device="cuda")
    for lo in range(0, n, 1 << 20):
        hi = min(n, lo + (1 << 20))
        c += Vm[:, lo:hi].double() @ g[lo:hi].double()
    fo.fosi_step(ctx, V, r_v, evals, g, None, mom, wa, sp)
    ctx.synchronize()
    c = c.cpu().numpy()
    gs = g[rows].double().cpu().numpy()
    w0s = w.w0[rows].double().cpu().numpy()
    # b = g - V c (zero initial momentum); e = V^T b computed the same way
    e = torch.zeros(r_v, dtype=torch.float64, device="cuda")
    for lo in range(0, n, 1 << 20):
        hi = min(n, lo + (1 << 20))
        vb = Vm[:, lo:hi].double()
        e += vb @ (g[lo:hi].double() - vb.T @ torch.from_numpy(c).cuda())
    e = e.cpu().numpy()
    al, lr = float(p.alpha), float(p.lr)
    b_s = gs - Vs @ c
    w_s = w0s - al * (Vs @ (c / evals)) - lr * b_s + lr * (Vs @ e)
    assert rel_l2(mom[rows].cpu().numpy(), b_s) <= 1e-5
    assert rel_l2(wa[rows].cpu().numpy(), w_s) <= 1e-5
    op.close()


def test_workload4_full_size(fo, ctx):
    """n = 25.6 M, r = 128, m = 80, k = 20, l = 10: the configuration bench.py times."""
    _full_size_planted(fo, ctx, 4)


def test_update_rules_at_four_million_rows(fo, ctx):
    """Both update rules (heavy ball and AdamW as base optimiser) with a dual variable at n = 4 M + 3 rows and 30
    columns, two consecutive steps each, against the complete oracle on the host: large enough that every sweep runs
    with the memory system under load and many workgroups in flight, small enough for the fp64 oracle (1 GB basis)."""
    n, r = (1 << 22) + 3, 30
    rng = np.random.default_rng(41)
    ld = wl.padded_ld(n)
    # an orthonormal basis without a 4 M x 30 QR: orthonormalise Gaussian columns by two rounds of Cholesky-QR in fp64
    A = rng.standard_normal((n, r))
    for _ in range(2):
        A = A @ np.linalg.inv(np.linalg.cholesky(A.T @ A).T)
    Vh = A.astype(np.float32)
    ev = np.concatenate([rng.uniform(1, 50, 20), -rng.uniform(0.5, 5, 10)])
    w0, g, b0 = (rng.standard_normal(n).astype(np.float32) for _ in range(3))
    pi = (0.1 * rng.standard_normal(n)).astype(np.float32)
    V = fo.ColMajor.from_numpy(Vh, ld)
    f32 = lambda x: float(np.float32(x))
    # heavy ball
    wd_, md_ = dev(w0), dev(b0)
    sp = fo.StepParams(0.1, 0.01, 0.9, 5e-4, 0)
    for _ in range(2):
        fo.fosi_step(ctx, V, r, ev, dev(g), dev(pi), md_, wd_, sp)
    ctx.synchronize()
    w_ref, b_ref = w0, b0
    for _ in range(2):
        w_ref, b_ref = oracle.fosi_step(w_ref, g, Vh, ev, b_ref, f32(0.1), f32(0.01), f32(0.9), f32(5e-4), pi=pi)
    assert rel_l2(wd_.cpu().numpy(), w_ref) <= 1e-5
    assert rel_l2(md_.cpu().numpy(), b_ref) <= 1e-5
    # AdamW
    ap = fo.AdamwParams(alpha=0.1, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.05, sigma=5e-4, curv_mode=0)
    wd_, m1, v1, work = dev(w0), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    for t in (1, 2):
        fo.fosi_step_adamw(ctx, V, r, ev, dev(g), dev(pi), m1, v1, work, wd_, t, ap)
    ctx.synchronize()
    w_ref, m_ref, v_ref = w0, np.zeros(n), np.zeros(n)
    for t in (1, 2):
        w_ref, m_ref, v_ref = oracle.fosi_step_adamw(w_ref, g, Vh, ev, m_ref, v_ref, t, f32(0.1), f32(1e-3), f32(0.9),
                                                     f32(0.999), f32(1e-8), f32(0.05), sigma=f32(5e-4), pi=pi)
    assert rel_l2(wd_.cpu().numpy(), w_ref) <= 1e-5
    assert rel_l2(m1.cpu().numpy(), m_ref) <= 1e-5
    assert rel_l2(v1.cpu().numpy(), v_ref) <= 1e-5


@pytest.mark.parametrize("mode_name", ["single", "twice", "selective"])
def test_workload4_other_schemes_full_size(fo, ctx, mode_name):
    """The printed single pass, the twice-repeated pass and the selective second pass at n = 25.6 M (40 steps): the
    first two run the kernel variants that keep computing with a stored value (sum of squares of the subtraction's
    output), the third switches its second pass on the device, at a size where the memory system is under full load.
    The tridiagonal must match the independent fp64 route."""
    from workloads.device import planted_workload_device
    w = planted_workload_device(4)
    n, r, m = w.n, w.r, 40
    U = fo.ColMajor(n, r, w.ld, buf=w.U)
    op = ctx.hvp_planted(U, w.lam, w.shift)
    Q = fo.ColMajor(n, m + 1, w.ld)
    Q.col(0).copy_(w.v1)
    mode = {"single": fo.REORTH_SINGLE, "twice": fo.REORTH_TWICE, "selective": fo.REORTH_SELECTIVE}[mode_name]
    alpha, beta, m_eff = fo.fosi_lanczos(ctx, op, Q, m, reorth_mode=mode)
    ctx.synchronize()
    assert m_eff == m and np.all(np.isfinite(alpha)) and np.all(np.isfinite(beta))
    if mode_name == "selective":
        # second pass exactly in the steps that cancelled much (a step within 2 % of the threshold may go either way)
        hn = np.sqrt(alpha ** 2 + np.concatenate([[0.0], beta[:-1]]) ** 2 + beta ** 2)
        thr = 2.0 ** -0.5
        sure, maybe = int(np.sum(beta / hn < 0.98 * thr)), int(np.sum(np.abs(beta / hn - thr) <= 0.02 * thr))
        assert sure <= fo.fosi_lanczos_second_passes(ctx) <= sure + maybe and sure >= m // 2
    lam = w.lam.cpu().numpy().astype(np.float64)
    scale = np.abs(lam).max()
    G = _gram_f64(w.U.view(r, w.ld), n, w.v1)
    a_ref, b_ref = reduced_tridiagonal_from_gram(G, lam, w.shift)
    assert np.max(np.abs(alpha[:m] - a_ref[:m])) < 1e-5 * scale
    assert np.max(np.abs(beta[: m - 1] - b_ref[: m - 1])) < 1e-5 * scale
    # orthonormal basis (the single pass drifts, cf. the scheme study; two passes stay at rounding level)
    Qm = Q.buf[: m * w.ld].view(m, w.ld)
    gram = torch.zeros(m, m, dtype=torch.float64, device="cuda")
    for lo in range(0, n, 1 << 20):
        blk = Qm[:, lo:min(n, lo + (1 << 20))].double()
        gram += blk @ blk.T
    dev_ = float((gram - torch.eye(m, dtype=torch.float64, device="cuda")).abs().max())
    assert dev_ < (1e-5 if mode_name == "single" else 1e-7), dev_
    op.close()


def test_workload5_full_size(fo, ctx):
    """n = 125 M, r = 128, m = 100, k = 20, l = 20: the largest block (138 GB of the 288 GB HBM)."""
    torch.cuda.empty_cache()
    _full_size_planted(fo, ctx, 5)
    torch.cuda.empty_cache()
