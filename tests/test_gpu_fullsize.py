"""GPU parity at the benchmark's sizes.

Workload 2 (n = 2^20) is small enough for the complete CPU oracle.  Workload 4
(n = 25.6 M, the configuration bench.py times) is too large for it, so the HIP
path is checked there through (a) the tridiagonal obtained by an independent
route (Householder reduction of the operator restricted to span([U, v1]), which
needs only a small Gram matrix, accumulated in float64 by library matmuls),
(b) invariants evaluated with library float64 operations, and (c) sampled rows
of the Ritz vectors and of the update, which the oracle's formulas give one by
one."""
import json

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from oracle.hvp import hvp_planted_chunked
from oracle.lanczos import tridiagonal
from tests.helpers import (reduced_ritz_coefficients, reduced_tridiagonal_from_gram, rel_l2,
                           sin_principal_angles, storage_emulation)

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
    # all m entries of the tridiagonal against the oracle run in the device's storage format (float64 arithmetic,
    # every stored vector rounded to fp32, two passes): the device may differ from that run by the order of its
    # float64 sums only, so the two must agree to 1e-3 of what the storage format itself costs
    emu = oracle.lanczos(lambda v: oracle.hvp_planted(w.U, w.lam, float(w.shift), v), w.v1, w.m, passes=2,
                         storage=np.float32)
    cost = np.maximum(np.abs(emu.alpha - res.alpha), np.abs(emu.beta - res.beta))
    diff = np.maximum(np.abs(alpha - emu.alpha), np.abs(beta - emu.beta))
    print("[workload 2] |T_fp32storage - T_float64|", np.array2string(cost, precision=1, max_line_width=100000))
    print("[workload 2] |T_gpu - T_fp32storage|   ", np.array2string(diff, precision=1, max_line_width=100000))
    assert np.all(diff <= 1e-3 * np.maximum.accumulate(cost))
    Qg = Q.to_numpy(w.m).astype(np.float64)
    print("[workload 2] max |Q_gpu - Q_fp32storage| by column",
          np.array2string(np.abs(Qg - emu.Q[:, : w.m]).max(axis=0), precision=1, max_line_width=100000))
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


def _deviation_from_reference(Vm, Um, v1, n, G, Cmat, k, l, chunk: int = 1 << 19) -> dict:
    """Deviation of the device's Ritz vectors (rows of Vm) from V_ref = [U, v1] Cmat (orthonormal columns), by
    library float64 operations on row chunks.  Returns the per-block principal-angle sines of the whole vectors
    and of their parts inside span([U, v1]), the per-pair norm of the part outside that span, and per pair how far
    the normalised in-span part leaves the reference block."""
    r_v, r = Vm.shape[0], Um.shape[0]
    dev_ = Vm.device
    C_t = torch.from_numpy(np.ascontiguousarray(Cmat)).to(dev_)
    R = np.linalg.cholesky(G).T                                   # [U, v1] = Bs R with orthonormal Bs
    Rinv_t = torch.from_numpy(np.linalg.inv(R)).to(dev_)
    blocks = {"top": slice(0, k), "bottom": slice(k, k + l)}

    def basis(lo, hi):
        return torch.cat([Um[:, lo:hi].double(), v1[lo:hi].double()[None, :]], dim=0).T     # rows x (r+1)

    cross = torch.zeros(r + 1, r_v, dtype=torch.float64, device=dev_)                       # [U, v1]^T V
    gram = torch.zeros(r_v, r_v, dtype=torch.float64, device=dev_)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        Vc = Vm[:, lo:hi].double().T
        cross += basis(lo, hi).T @ Vc
        gram += Vc.T @ Vc
    Y = Rinv_t.T @ cross                                          # Bs^T V: in-span coordinates
    W = C_t.T @ cross                                             # V_ref^T V
    e_out = torch.zeros(r_v, dtype=torch.float64, device=dev_)
    e_blk = {name: torch.zeros(b.stop - b.start, b.stop - b.start, dtype=torch.float64, device=dev_)
             for name, b in blocks.items()}
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        Bc = basis(lo, hi)
        Vc = Vm[:, lo:hi].double().T
        out = Vc - (Bc @ Rinv_t) @ Y
        e_out += (out * out).sum(dim=0)
        Vref = Bc @ C_t
        for name, b in blocks.items():
            if b.stop > b.start:
                E = Vc[:, b] - Vref[:, b] @ W[b, b]
                e_blk[name] += E.T @ E
    gram_h, Y_h = gram.cpu().numpy(), Y.cpu().numpy()
    Cref = R @ Cmat
    res = {"out_norm": np.sqrt(e_out.cpu().numpy() / np.diag(gram_h)), "total_sin": {}, "in_span_sin": {},
           "in_span_leave": np.zeros(r_v)}
    for name, b in blocks.items():
        if b.stop == b.start:
            continue
        L = np.linalg.cholesky(gram_h[b, b])
        Li = np.linalg.inv(L)
        res["total_sin"][name] = float(np.sqrt(max(0.0, np.linalg.eigvalsh(Li @ e_blk[name].cpu().numpy() @ Li.T).max())))
        res["in_span_sin"][name] = float(sin_principal_angles(Cref[:, b], Y_h[:, b]).max())
        A = np.linalg.qr(Cref[:, b])[0]
        Yb = Y_h[:, b] / np.linalg.norm(Y_h[:, b], axis=0)
        res["in_span_leave"][b] = np.linalg.norm(Yb - A @ (A.T @ Yb), axis=0)
    return res


def _full_size_planted(fo, ctx, cfg_id, w=None):
    from workloads.device import planted_workload_device
    if w is None:
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

    # Reference: the independent fp64 route (Householder reduction of the operator restricted to span([U, v1]), from
    # the Gram matrix of [U, v1] accumulated by library float64 matmuls): the whole tridiagonal, the Ritz values and
    # the Ritz vectors V_ref = [U, v1] Cmat.
    # Bars: the tolerances the workloads state (Ritz values 1e-4 relative, principal angles 1e-3 rad) wherever an
    # implementation with fp32 vectors can meet them, and otherwise twice what the CPU emulation of the storage
    # format shows for THIS problem: the oracle's recurrence, float64 arithmetic, every stored vector rounded to
    # fp32, run on two 65 536-row embeddings of this instance's restricted problem (tests/helpers.storage_emulation;
    # tests/test_fp32_storage_emulation.py pins what that emulation finds and why).
    G = _gram_f64(w.U.view(r, w.ld), n, w.v1)
    a_ref, b_ref = reduced_tridiagonal_from_gram(G, lam, w.shift)
    ev_ref, Cmat, resid_ref, all_ref = reduced_ritz_coefficients(G, lam, w.shift, m, w.k, w.l)
    emus = [storage_emulation(G, lam, w.shift, m, w.k, w.l, n_rows=1 << 16, seed=sd) for sd in (0, 1)]
    emu = {key: np.maximum(emus[0][key], emus[1][key]) for key in ("value_abs_err", "out_norm", "in_span_leave", "dT")}
    for key in ("total_sin", "in_span_sin"):
        emu[key] = {b: max(e[key][b] for e in emus) for b in emus[0][key]}
    assert np.max(np.abs(emus[0]["evals"] - ev_ref)) < 1e-8 * scale     # the emulation runs this very problem

    # (a) the whole tridiagonal, all m entries of both diagonals: within twice the emulated deviation, taken as an
    # envelope (largest deviation up to that index, since the recurrence carries its errors forward)
    dT = np.maximum(np.abs(alpha - a_ref[:m]), np.abs(beta - b_ref[:m]))
    envelope = np.maximum.accumulate(emu["dT"])
    print(f"[workload {cfg_id}] |T_gpu - T_ref| by index {np.array2string(dT, precision=1, max_line_width=100000)}")
    print(f"[workload {cfg_id}] emulated envelope    {np.array2string(envelope, precision=1, max_line_width=100000)}")
    assert np.all(dT <= 2.0 * envelope), np.flatnonzero(dT > 2.0 * envelope)

    # (b) Ritz values: 1e-4 relative, or twice the emulated error of that pair
    err = np.abs(evals - ev_ref)
    resolved_all = resid_ref <= 1e-2 * np.abs(ev_ref)
    print(f"[workload {cfg_id}] Ritz value errors {np.array2string(err, precision=1, max_line_width=100000)}; emulated "
          f"{np.array2string(emu['value_abs_err'], precision=1, max_line_width=100000)}; resolved by the reference: "
          f"{resolved_all.sum()} of {r_v}")
    assert resolved_all.sum() >= w.k
    assert np.max(err[resolved_all] / np.abs(ev_ref[resolved_all])) <= 1e-4
    assert np.all(err <= np.maximum(1e-4 * np.abs(ev_ref), 2.0 * emu["value_abs_err"]))

    # (c) Ritz vectors against V_ref, evaluated in float64 row chunk by row chunk (differences are formed element by
    # element, so angles far below 1e-8 rad are resolved).  Three figures: the principal angles of each block as
    # whole vectors; the norm of each Ritz vector's component outside span([U, v1]) -- rounding noise inside the
    # (n - r)-dimensional eigenspace of the shift, where every direction is an exact eigenvector, so that part is
    # valid but not unique; and the principal angles of the in-span parts, which are unique.
    Vm_ = V.buf[: r_v * w.ld].view(r_v, w.ld)
    Um_ = w.U.view(r, w.ld)
    dev_rep = _deviation_from_reference(Vm_, Um_, w.v1, n, G, Cmat, w.k, w.l)
    record = {"workload": cfg_id, "n": n, "m": m, "evals_ref": ev_ref, "resid_ref": resid_ref, "value_abs_err": err,
              "out_norm": dev_rep["out_norm"], "in_span_leave": dev_rep["in_span_leave"],
              "total_sin": dev_rep["total_sin"], "in_span_sin": dev_rep["in_span_sin"], "dT": dT,
              "emulated": emu}
    print("PARITY_RECORD " + json.dumps(record, default=lambda o: np.asarray(o).tolist()))
    for name in dev_rep["total_sin"]:
        print(f"[workload {cfg_id}] {name} block: whole-vector sin {dev_rep['total_sin'][name]:.2e} (emulated "
              f"{emu['total_sin'][name]:.2e}), in-span sin {dev_rep['in_span_sin'][name]:.2e} (emulated "
              f"{emu['in_span_sin'][name]:.2e})")
        assert dev_rep["total_sin"][name] <= max(1e-3, 2.0 * emu["total_sin"][name])
        assert dev_rep["in_span_sin"][name] <= max(1e-3, 2.0 * emu["in_span_sin"][name])
    print(f"[workload {cfg_id}] out-of-span norm per pair {np.array2string(dev_rep['out_norm'], precision=1, max_line_width=100000)}; "
          f"emulated {np.array2string(emu['out_norm'], precision=1, max_line_width=100000)}")
    # per pair; the emulation forms its Ritz vectors in float64 and rounds them once, the device accumulates the m
    # products of V = Q S in fp32: up to u32 sqrt(m) more (measured ~1e-7, and only visible on the converged pairs)
    assert np.all(dev_rep["out_norm"] <= 2.0 * emu["out_norm"] + 2.0 ** -24 * np.sqrt(m))
    moved = np.hypot(dev_rep["out_norm"], dev_rep["in_span_leave"])
    assert moved[resolved_all].max() < 1e-3                       # every pair the reference has resolved: the stated bar

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


@pytest.mark.parametrize("mode_name", ["single", "twice"])
def test_in_place_rewrites_at_three_million_rows(fo, ctx, mode_name):
    """The schemes whose subtraction sweep rewrites the vector in place with the hand-written write-through store and
    then goes on computing with the stored values (sum of squares), at a size where thousands of workgroups are in
    flight and the rows are ragged (3 * 2^20 + 1): EVERY element of the first ten Lanczos vectors against the
    oracle.  (That store once lost elements under memory pressure -- its data registers were overwritten inside
    the hardware's wait states -- and only the 8 GB full-size runs noticed.)"""
    n, m = 3 * (1 << 20) + 1, 10
    w = wl.planted_workload(2, n=n)
    ld = wl.padded_ld(n)
    U = fo.ColMajor.from_numpy(w.U, ld)
    op = ctx.hvp_planted(U, dev(w.lam), float(w.shift))
    Q = fo.ColMajor(n, m + 1, ld)
    Q.col(0).copy_(dev(w.v1))
    mode = {"single": fo.REORTH_SINGLE, "twice": fo.REORTH_TWICE}[mode_name]
    alpha, beta, m_eff = fo.fosi_lanczos(ctx, op, Q, m, reorth_mode=mode)
    ctx.synchronize()
    assert m_eff == m
    res = oracle.lanczos(lambda v: hvp_planted_chunked(w.U, w.lam, float(w.shift), v), w.v1, m,
                         passes=1 if mode_name == "single" else 2)
    Qg = Q.to_numpy(m + 1).astype(np.float64)
    assert np.all(np.isfinite(Qg))
    for j in range(m + 1):
        tol = 1e-4 * np.abs(res.Q[:, j]).max()
        bad = np.flatnonzero(np.abs(Qg[:, j] - res.Q[:, j]) > tol)
        assert bad.size == 0, (mode_name, j, bad[:8], bad.size)
    scale = np.abs(w.lam).max()
    assert np.max(np.abs(alpha - res.alpha)) < 1e-6 * scale and np.max(np.abs(beta - res.beta)) < 1e-6 * scale
    op.close()


@pytest.fixture(scope="module")
def w5():
    """The largest block (n = 125 M, 64 GB of planted eigenvectors), generated once for the tests below."""
    from workloads.device import planted_workload_device
    torch.cuda.empty_cache()
    w = planted_workload_device(5)
    yield w
    del w
    torch.cuda.empty_cache()


def test_workload5_full_size(fo, ctx, w5):
    """n = 125 M, r = 128, m = 100, k = 20, l = 20: the largest block (138 GB of the 288 GB HBM)."""
    _full_size_planted(fo, ctx, 5, w5)
    torch.cuda.empty_cache()


def test_workload5_whole_schedule(fo, ctx, w5):
    """The largest workload as it is stated: one hundred updates with the curvature refreshed every ten, i.e. ten
    outer iterations of Algorithm 3 at n = 125 M -- Lanczos (m = 100) from a fresh seeded start vector, Ritz
    extraction (20 + 20), w = w_a + pi / sigma, ten updates by Eq. 14 with the dual variable and fresh gradients,
    pi += sigma (w_a - w) (Eq. 11) -- with the momentum and the multiplier carried over.  Reference: the same
    equations in float64 over the full vectors (tests/helpers.Float64State, pinned against the oracle on the CPU),
    evaluated on the device's own Ritz pairs of each refresh; everything else (anchor, dual variable, momentum,
    parameters) is the reference's own, so the comparison runs end to end over all hundred updates."""
    import time

    from tests.helpers import Float64State
    w = w5
    n, m, r, r_v = w.n, w.m, w.r, w.k + w.l
    p = w.params
    sig, al, lr, mu = float(p.sigma), float(p.alpha), float(p.lr), float(p.momentum)
    sp = fo.StepParams(al, lr, mu, sig, 0)
    U = fo.ColMajor(n, r, w.ld, buf=w.U)
    op = ctx.hvp_planted(U, w.lam, w.shift)
    Q = fo.ColMajor(n, m + 1, w.ld)
    V = fo.ColMajor(n, r_v, w.ld)
    Vm = V.buf[: r_v * w.ld].view(r_v, w.ld)[:, :n]
    wa = w.w0.clone()
    pi, mom, anchor = (torch.zeros(n, device="cuda") for _ in range(3))
    ref = Float64State(w.w0)
    gen = torch.Generator(device="cuda")
    t_gpu = 0.0
    for outer in range(10):
        gen.manual_seed(5_000 + outer)
        Q.col(0).copy_(torch.randn(n, generator=gen, device="cuda", dtype=torch.float32))
        grads = [w.grad(10 * outer + t) for t in range(w.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        alpha, beta, m_eff = fo.fosi_lanczos(ctx, op, Q, m)
        evals, _ = fo.fosi_ritz(ctx, Q, m_eff, alpha, beta, w.k, w.l, V)
        fo.fosi_admm_begin(ctx, sig, pi, anchor, wa)
        for t in range(w.steps):
            fo.fosi_step(ctx, V, r_v, evals, grads[t], pi, mom, wa, sp)
        fo.fosi_admm_end(ctx, sig, anchor, wa, pi)
        ctx.synchronize()
        t_gpu += time.perf_counter() - t0
        assert m_eff == m
        ref.begin(sig)
        for t in range(w.steps):
            ref.step(Vm, evals, grads[t], al, lr, mu, sig)
        ref.end(sig)
        del grads
        rel = lambda a, b: float((a.double() - b).norm() / b.norm())
        e_anchor, e_w, e_b = rel(anchor, ref.anchor), rel(wa, ref.w), rel(mom, ref.b)
        e_pi = float((pi.double() - ref.pi).norm())
        bound_pi = 8 * sig * float(ref.w.norm()) * 2.0 ** -24 * (outer + 1)
        print(f"[workload 5 schedule] outer {outer}: rel L2 anchor {e_anchor:.1e}, w_a {e_w:.1e}, momentum {e_b:.1e}; "
              f"|pi - pi_ref| {e_pi:.2e} (bound {bound_pi:.2e}, |pi_ref| {float(ref.pi.norm()):.2e})", flush=True)
        assert e_anchor <= 1e-5 and e_w <= 1e-5, outer
        assert e_b <= 5e-5, outer
        # the multiplier is sigma times a difference of two stored fp32 vectors of size |w|: its error is measured
        # against sigma |w| 2^-24, the rounding of those vectors, not against its own (small) size
        assert e_pi <= bound_pi, outer
    print(f"[workload 5 schedule] 10 outer iterations (100 updates, 10 curvature refreshes): {t_gpu:.2f} s on the device",
          flush=True)
    op.close()
    del ref
    torch.cuda.empty_cache()
