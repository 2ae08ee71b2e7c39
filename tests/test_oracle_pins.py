"""Pins for the CPU oracle: every check here compares the oracle with something
it does not compute itself (planted eigenvalues, a dense eigensolver, LAPACK's
Householder tridiagonalisation, a library SGD, autograd, closed forms)."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle.lanczos import lanczos_row_sharded, tridiagonal
from tests.helpers import reduced_ritz_coefficients, reduced_tridiagonal, rel_l2, sin_principal_angles


def planted_op(w):
    return lambda v: oracle.hvp_planted(w.U, w.lam, float(w.shift), v)


def make_cfg1():
    w = wl.planted_workload(1)
    res = oracle.lanczos(planted_op(w), w.v1, w.m)
    return w, res


def make_cfg2_small():
    w = wl.planted_workload(2, n=1 << 15)
    res = oracle.lanczos(planted_op(w), w.v1, w.m)
    return w, res


def make_ggn_small():
    return wl.ggn_workload(B=16, d=8, C=5)


# (plain builders above so that tests/test_pins_catch_planted_mistakes.py can rebuild the inputs
# with a deliberately broken oracle)
@pytest.fixture(scope="module")
def cfg1():
    return make_cfg1()


@pytest.fixture(scope="module")
def cfg2_small():
    return make_cfg2_small()


# ---------------------------------------------------------------- operators
def test_hvp_planted_matches_dense_matrix():
    w = wl.planted_workload(1, n=300)
    U = w.U.astype(np.float64)
    H = U @ np.diag(w.lam.astype(np.float64)) @ U.T + float(w.shift) * np.eye(300)
    v = wl.normal_vector(1, 77, 300)
    assert rel_l2(oracle.hvp_planted(w.U, w.lam, w.shift, v), H @ v) < 1e-13
    from oracle.hvp import hvp_planted_chunked
    assert rel_l2(hvp_planted_chunked(w.U, w.lam, w.shift, v, rows=64), H @ v) < 1e-13


def test_hvp_planted_eigenvectors():
    # U's own columns are eigenvectors with eigenvalue lam_j + shift (U is orthonormal to fp32 rounding)
    w = wl.planted_workload(1)
    for j in (0, 7, 31):
        u = w.U[:, j].astype(np.float64)
        hv = oracle.hvp_planted(w.U, w.lam, w.shift, u)
        assert rel_l2(hv, (float(w.lam[j]) + float(w.shift)) * u) < 1e-6


# ---------------------------------------------------------------- Lanczos
def test_start_vector_is_normalised(cfg1):
    w, res = cfg1
    v = w.v1.astype(np.float64)
    assert np.allclose(res.Q[:, 0], v / np.sqrt(v @ v), rtol=0, atol=1e-15)


def test_breakdown_at_exhausted_krylov_space(cfg1):
    # rank-32 plus a multiple of the identity: the Krylov space has dimension 33 < m = 40
    _, res = cfg1
    assert res.m_eff == 33


def test_planted_spectrum_top_values(cfg1, cfg2_small):
    for w, res in (cfg1, cfg2_small):
        rz = oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, w.k, w.l)
        truth = np.sort(w.lam.astype(np.float64))[::-1][: w.k] + float(w.shift)
        conv = rz.resid[: w.k] <= 1e-8 * np.abs(rz.evals[: w.k])
        assert conv.all()
        # U is orthonormal only up to its fp32 storage (1e-8), which moves the eigenvalues by ~1e-8 ||H||
        assert np.max(np.abs(rz.evals[: w.k] - truth) / truth) < 1e-7


def test_planted_spectrum_bottom_values(cfg2_small):
    w, res = cfg2_small
    rz = oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, w.k, w.l)
    truth = np.sort(w.lam.astype(np.float64))[: w.l] + float(w.shift)
    got = rz.evals[w.k:]
    conv = rz.resid[w.k:] <= 1e-6
    assert conv.sum() >= 3
    assert np.max(np.abs(got[conv] - truth[conv])) < 1e-5
    assert np.all(np.diff(got) > 0) and np.all(np.diff(rz.evals[: w.k]) < 0)   # ordering convention


def test_tridiagonal_matches_householder_reduction(cfg1, cfg2_small):
    for w, res in (cfg1, cfg2_small):
        a, b = reduced_tridiagonal(w.U, w.lam, w.shift, w.v1)
        me = res.m_eff
        scale = np.abs(w.lam).max()
        assert np.max(np.abs(a[:me] - res.alpha[:me])) < 1e-12 * scale
        assert np.max(np.abs(b[: me - 1] - res.beta[: me - 1])) < 1e-12 * scale


def test_ritz_pairs_match_householder_route(cfg2_small):
    # Ritz values *and vectors* (converged or not) from the restricted problem, reduced by Householder reflectors
    w, res = cfg2_small
    rz = oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, w.k, w.l)
    B = np.column_stack([w.U.astype(np.float64), w.v1.astype(np.float64)])
    ev, Cm, resid, _ = reduced_ritz_coefficients(B.T @ B, w.lam, w.shift, w.m, w.k, w.l)
    assert np.allclose(resid, rz.resid, rtol=1e-6, atol=1e-9)
    assert np.max(np.abs(ev - rz.evals)) < 1e-9 * np.abs(w.lam).max()
    assert sin_principal_angles(rz.V[:, : w.k], (B @ Cm)[:, : w.k]).max() < 1e-8
    assert sin_principal_angles(rz.V[:, w.k:], (B @ Cm)[:, w.k:]).max() < 1e-8


def test_lanczos_invariants(cfg2_small):
    w, res = cfg2_small
    me = res.m_eff
    Q = res.Q[:, :me]
    assert np.abs(Q.T @ Q - np.eye(me)).max() < 1e-8
    T = tridiagonal(res.alpha, res.beta, me)
    HQ = np.column_stack([planted_op(w)(Q[:, j]) for j in range(me)])
    R = HQ - Q @ T
    R[:, me - 1] -= res.beta[me - 1] * res.Q[:, me]
    assert np.linalg.norm(R) / np.abs(w.lam).max() < 1e-8
    # Eq. 5 / Eq. 6 entry by entry
    for i in (0, 5, me - 2):
        assert abs(Q[:, i] @ HQ[:, i] - res.alpha[i]) < 1e-8 * np.abs(w.lam).max()
        assert abs(Q[:, i + 1] @ HQ[:, i] - res.beta[i]) < 1e-8 * np.abs(w.lam).max()
    # Ritz values are Rayleigh quotients and lie inside the spectrum
    rz = oracle.ritz(res.Q, res.alpha, res.beta, me, w.k, w.l)
    for j in range(w.k + w.l):
        y = rz.V[:, j]
        assert abs(y @ planted_op(w)(y) - rz.evals[j]) < 1e-7 * np.abs(w.lam).max()
    lo, hi = w.lam.min() + float(w.shift), w.lam.max() + float(w.shift)
    assert rz.all_evals.min() >= lo - 1e-6 and rz.all_evals.max() <= hi + 1e-6 * hi
    # Cauchy interlacing between m-1 and m steps
    u_small = np.linalg.eigvalsh(tridiagonal(res.alpha, res.beta, me - 1))
    u_big = rz.all_evals
    assert np.all(u_big[:-1] <= u_small + 1e-9 * hi) and np.all(u_small <= u_big[1:] + 1e-9 * hi)


def test_dense_bruteforce_cfg1(cfg1):
    w, res = cfg1
    U = w.U.astype(np.float64)
    H = U @ np.diag(w.lam.astype(np.float64)) @ U.T + float(w.shift) * np.eye(w.n)
    ev, evec = np.linalg.eigh(H)
    rz = oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, w.k, w.l)
    assert np.max(np.abs(rz.evals - ev[::-1][: w.k]) / ev[::-1][: w.k]) < 1e-10
    s = sin_principal_angles(evec[:, ::-1][:, : w.k], rz.V)
    assert s.max() < 1e-7
    # with the whole invariant subspace captured every Ritz value is an eigenvalue of H
    assert np.max(np.abs(np.sort(rz.all_evals)[1:] - ev[-32:])) < 1e-6


def test_full_spectrum_of_small_diagonal_operator():
    n = 48
    d = np.linspace(-3.0, 7.0, n) + 0.01 * np.arange(n) ** 1.5
    v1 = wl.normal_vector(1, 99, n)
    res = oracle.lanczos(lambda v: oracle.hvp_diag(d, v), v1, n, passes=2, breakdown_tol=1e-12)
    assert res.m_eff == n
    u = np.linalg.eigvalsh(tridiagonal(res.alpha, res.beta, n))
    assert np.max(np.abs(u - np.sort(d))) < 1e-8


def test_second_pass_changes_nothing_in_float64(cfg2_small):
    w, res = cfg2_small
    res2 = oracle.lanczos(planted_op(w), w.v1, 30, passes=2)
    assert np.max(np.abs(res2.alpha[:30] - res.alpha[:30])) < 1e-8 * np.abs(w.lam).max()
    assert np.max(np.abs(res2.beta[:29] - res.beta[:29])) < 1e-8 * np.abs(w.lam).max()


def test_row_sharded_algorithm_reproduces_single_device(cfg1):
    w, res = cfg1
    for C in (2, 5):
        sh = lanczos_row_sharded(planted_op(w), w.v1, w.m, C)
        assert sh.m_eff == res.m_eff
        me = res.m_eff
        assert np.max(np.abs(sh.alpha[:me] - res.alpha[:me])) < 1e-9 * 1e3
        assert np.max(np.abs(sh.beta[: me - 1] - res.beta[: me - 1])) < 1e-9 * 1e3


def test_ritz_argument_checks(cfg1):
    _, res = cfg1
    with pytest.raises(ValueError):
        oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, 30, 10)
    with pytest.raises(ValueError):
        oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, 0, 0)


# ---------------------------------------------------------------- update rule
def _orthonormal(n, r, seed):
    return np.linalg.qr(np.random.default_rng(seed).standard_normal((n, r)))[0]


def test_step_closed_form_on_coordinate_subspace():
    n, r = 40, 6
    rng = np.random.default_rng(1)
    V = np.eye(n)[:, :r]
    a = np.array([5.0, 3.0, 2.0, -1.5, 0.7, 0.2])
    w, g, b = rng.standard_normal(n), rng.standard_normal(n), rng.standard_normal(n)
    al, lr, mu = 0.3, 0.05, 0.8
    w1, b1 = oracle.fosi_step(w, g, V, a, b, al, lr, mu)
    exp_w = w.copy()
    exp_w[:r] += -al * g[:r] / a                     # Newton step coordinate-wise
    exp_b = mu * b
    exp_b[r:] += g[r:]                               # momentum buffer gets the complement part of g
    exp_w[r:] += -lr * exp_b[r:]                     # and the base step is re-projected
    assert np.allclose(w1, exp_w, atol=1e-14) and np.allclose(b1, exp_b, atol=1e-14)
    w2, _ = oracle.fosi_step(w, g, V, a, b, al, lr, mu, curv_mode="abs")
    exp_w[:r] = w[:r] - al * g[:r] / np.abs(a)
    assert np.allclose(w2, exp_w, atol=1e-14)


def test_step_without_subspace_is_library_sgd_momentum():
    import torch
    n = 64
    rng = np.random.default_rng(2)
    w = rng.standard_normal(n)
    p = torch.nn.Parameter(torch.tensor(w, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=0.01, momentum=0.9)
    b = np.zeros(n)
    V = np.zeros((n, 0))
    for t in range(5):
        g = rng.standard_normal(n)
        w, b = oracle.fosi_step(w, g, V, np.zeros(0), b, 0.1, 0.01, 0.9)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        assert np.allclose(w, p.detach().numpy(), atol=1e-14)


def test_step_orthogonality_and_zero_momentum():
    n, r = 200, 7
    V = _orthonormal(n, r, 3)
    rng = np.random.default_rng(4)
    a = rng.uniform(0.5, 9.0, r)
    w, g, b = rng.standard_normal(n), rng.standard_normal(n), rng.standard_normal(n)
    # momentum 0: Delta_2 = -lr (I - V V^T) g, Delta_1 = -alpha V diag(1/a) V^T g
    w1, _ = oracle.fosi_step(w, g, V, a, b, 0.2, 0.03, 0.0)
    d1 = -0.2 * V @ ((V.T @ g) / a)
    d2 = -0.03 * (g - V @ (V.T @ g))
    assert np.allclose(w1 - w, d1 + d2, atol=1e-13)
    assert abs(d1 @ d2) < 1e-13
    # with momentum: the part of the update outside Delta_1 stays orthogonal to V
    w2, _ = oracle.fosi_step(w, g, V, a, b, 0.2, 0.03, 0.9)
    assert np.abs(V.T @ (w2 - w - d1)).max() < 1e-13


def test_step_solves_quadratic_in_subspace_in_one_step():
    n, r = 120, 5
    V = _orthonormal(n, r, 5)
    a = np.array([9.0, 4.0, 2.5, 1.0, 0.3])
    w = np.random.default_rng(6).standard_normal(n)
    g = V @ (a * (V.T @ w))                           # gradient of 0.5 w^T V diag(a) V^T w
    w1, _ = oracle.fosi_step(w, g, V, a, np.zeros(n), 1.0, 0.01, 0.9)
    assert np.abs(V.T @ w1).max() < 1e-13


def test_step_with_zero_dual_equals_plain_step():
    n, r = 90, 4
    V = _orthonormal(n, r, 7)
    rng = np.random.default_rng(8)
    a = rng.uniform(1, 5, r)
    w, g, b = rng.standard_normal(n), rng.standard_normal(n), rng.standard_normal(n)
    plain = oracle.fosi_step(w, g, V, a, b, 0.1, 0.01, 0.9)
    dual0 = oracle.fosi_step(w, g, V, a, b, 0.1, 0.01, 0.9, sigma=0.0, pi=np.zeros(n))
    assert np.array_equal(plain[0], dual0[0]) and np.array_equal(plain[1], dual0[1])


def test_step_with_dual_closed_form_and_g1_readings():
    n, r = 90, 4
    V = _orthonormal(n, r, 9)
    rng = np.random.default_rng(10)
    a = rng.uniform(1, 5, r)
    w, g, b0, pi = (rng.standard_normal(n) for _ in range(4))
    b0 = b0 - V @ (V.T @ b0)
    sig, al, lr, mu = 0.05, 0.1, 0.01, 0.9
    w1, b1 = oracle.fosi_step(w, g, V, a, b0, al, lr, mu, sigma=sig, pi=pi)
    gt = g + pi
    Pc = np.eye(n) - V @ V.T
    exp = w - al * V @ np.diag(1.0 / (a + sig)) @ V.T @ gt - lr * Pc @ (mu * b0 + Pc @ gt)
    assert np.allclose(w1, exp, atol=1e-13)
    # the two readings of "g_1" in Eq. 14 give the same update for a linear base optimiser and fixed V
    w2, b2 = oracle.fosi_step(w, g, V, a, b0, al, lr, mu, sigma=sig, pi=pi, g1_reading="literal")
    assert np.allclose(w1, w2, atol=1e-13)
    assert not np.allclose(b1, b2, atol=1e-6)         # ... but not the same momentum buffer


def test_step_abs_mode_with_dual_and_negative_curvature():
    # negative and tiny Ritz values with a penalty: signed divides by a + sigma, abs by |a| + sigma (not |a + sigma|)
    n, r = 70, 4
    V = _orthonormal(n, r, 21)
    rng = np.random.default_rng(22)
    a = np.array([3.0, -2.0, 0.5, -0.01])
    w, g, b0, pi = (rng.standard_normal(n) for _ in range(4))
    sig, al, lr, mu = 0.05, 0.3, 0.02, 0.7
    gt = g + pi
    Pc = np.eye(n) - V @ V.T
    tail = -lr * Pc @ (mu * b0 + Pc @ gt)
    w_signed, _ = oracle.fosi_step(w, g, V, a, b0, al, lr, mu, sigma=sig, pi=pi)
    assert np.allclose(w_signed, w - al * V @ ((V.T @ gt) / np.array([3.05, -1.95, 0.55, 0.04])) + tail, atol=1e-12)
    w_abs, _ = oracle.fosi_step(w, g, V, a, b0, al, lr, mu, sigma=sig, pi=pi, curv_mode="abs")
    assert np.allclose(w_abs, w - al * V @ ((V.T @ gt) / np.array([3.05, 2.05, 0.55, 0.06])) + tail, atol=1e-12)


def test_adamw_step_dense_closed_form():
    """Three consecutive updates with a non-empty subspace, a dual variable and both curvature modes: the base
    optimiser's vector is taken from torch.optim.AdamW fed with the complement part of g + pi, the projections are
    dense matrices."""
    import torch
    n, r = 80, 5
    V = _orthonormal(n, r, 23)
    rng = np.random.default_rng(24)
    a = np.array([4.0, 1.5, -0.8, 0.3, -0.02])
    lr, b1, b2, eps, wd, al, sig = 2e-3, 0.9, 0.99, 1e-8, 0.1, 0.25, 0.05
    Pc = np.eye(n) - V @ V.T
    for mode, denom in (("signed", a + sig), ("abs", np.abs(a) + sig)):
        w = rng.standard_normal(n)
        m, v = np.zeros(n), np.zeros(n)
        p = torch.nn.Parameter(torch.tensor(w, dtype=torch.float64))
        opt = torch.optim.AdamW([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
        for t in range(1, 4):
            g, pi = rng.standard_normal(n), 0.3 * rng.standard_normal(n)
            with torch.no_grad():
                p.copy_(torch.tensor(w))                      # the library optimiser starts from the current point
            p.grad = torch.tensor(Pc @ (g + pi))
            opt.step()
            o = p.detach().numpy() - w                        # its whole descent vector, decay included
            expect = w - al * V @ ((V.T @ (g + pi)) / denom) + Pc @ o
            w, m, v = oracle.fosi_step_adamw(w, g, V, a, m, v, t, al, lr, b1, b2, eps, wd, sigma=sig, pi=pi, curv_mode=mode)
            assert np.allclose(w, expect, rtol=0, atol=1e-12)


def test_adamw_step_without_subspace_is_library_adamw():
    import torch
    n = 64
    rng = np.random.default_rng(12)
    w = rng.standard_normal(n)
    p = torch.nn.Parameter(torch.tensor(w, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.05)
    m, v = np.zeros(n), np.zeros(n)
    V = np.zeros((n, 0))
    for t in range(1, 6):
        g = rng.standard_normal(n)
        w, m, v = oracle.fosi_step_adamw(w, g, V, np.zeros(0), m, v, t, 0.1, 1e-3, 0.9, 0.999, 1e-8, 0.05)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        assert np.allclose(w, p.detach().numpy(), rtol=0, atol=1e-13)


def test_adamw_step_structure():
    n, r = 150, 5
    V = _orthonormal(n, r, 13)
    rng = np.random.default_rng(14)
    a = rng.uniform(1, 8, r)
    w, g, pi = rng.standard_normal(n), rng.standard_normal(n), 0.1 * rng.standard_normal(n)
    w1, m1, v1 = oracle.fosi_step_adamw(w, g, V, a, np.zeros(n), np.zeros(n), 1, 0.2, 1e-3, 0.9, 0.999, 1e-8, 0.05,
                                        sigma=0.05, pi=pi)
    d1 = -0.2 * V @ ((V.T @ (g + pi)) / (a + 0.05))
    # everything besides the Newton part is orthogonal to V; the moments only see the complement of g + pi
    assert np.abs(V.T @ (w1 - w - d1)).max() < 1e-15
    x = (g + pi) - V @ (V.T @ (g + pi))
    assert np.allclose(m1, 0.1 * x, atol=1e-15) and np.allclose(v1, 0.001 * x * x, atol=1e-15)
    # first step, no decay: the optimiser's vector is -lr sign(x) up to eps, re-projected
    w2, _, _ = oracle.fosi_step_adamw(w, g, V, a, np.zeros(n), np.zeros(n), 1, 0.2, 1e-3, 0.9, 0.999, 1e-12, 0.0)
    x0 = g - V @ (V.T @ g)
    o = -1e-3 * np.sign(x0)
    d1b = -0.2 * V @ ((V.T @ g) / a)
    assert np.allclose(w2 - w - d1b, o - V @ (V.T @ o), atol=1e-9)


# ---------------------------------------------------------------- ADMM outer
def test_admm_outer_rules():
    n = 50
    rng = np.random.default_rng(11)
    wa, pi = rng.standard_normal(n), rng.standard_normal(n)
    sig = 5e-4
    anchor, wa0 = oracle.admm_begin(wa, pi, sig)
    assert np.allclose(anchor, wa + pi / sig) and np.array_equal(anchor, wa0)
    moved = wa0 + rng.standard_normal(n)
    pi1 = oracle.admm_end(anchor, moved, pi, sig)
    assert np.allclose(pi1, pi + sig * (moved - anchor))
    # first outer with pi = 0: the anchor is the old point; next anchor = w_a + (w_a - w_prev)
    a0, w0 = oracle.admm_begin(wa, np.zeros(n), sig)
    assert np.array_equal(a0, wa)
    w_after = w0 + rng.standard_normal(n)
    p1 = oracle.admm_end(a0, w_after, np.zeros(n), sig)
    a1, _ = oracle.admm_begin(w_after, p1, sig)
    assert np.allclose(a1, w_after + (w_after - wa), atol=1e-12)


# ---------------------------------------------------------------- softmax GGN
@pytest.fixture(scope="module")
def ggn_small():
    return make_ggn_small()


def test_ggn_equals_autograd_hessian_product(ggn_small):
    import torch
    g = ggn_small
    X = torch.tensor(g.X, dtype=torch.float64)
    y = torch.tensor(g.labels)
    W = torch.tensor(g.W, dtype=torch.float64)

    def loss(Wm):
        return torch.nn.functional.cross_entropy(X @ Wm, y)

    v = wl.normal_vector(3, 50, g.n).astype(np.float64)
    _, hv = torch.autograd.functional.hvp(loss, W, torch.tensor(v).reshape(g.d, g.C))
    assert rel_l2(oracle.hvp_softmax_ggn(g.X, g.W, v), hv.reshape(-1).numpy()) < 1e-12


def test_ggn_dense_kronecker_sum(ggn_small):
    g = ggn_small
    X, W = g.X.astype(np.float64), g.W.astype(np.float64)
    P = oracle.softmax_rows(X @ W)
    H = np.zeros((g.n, g.n))
    for b in range(g.B):
        H += np.kron(np.outer(X[b], X[b]), np.diag(P[b]) - np.outer(P[b], P[b])) / g.B
    v = wl.normal_vector(3, 51, g.n)
    assert rel_l2(oracle.hvp_softmax_ggn(g.X, g.W, v), H @ v.astype(np.float64)) < 1e-12
    assert np.linalg.eigvalsh(H).min() > -1e-12                 # PSD
    assert np.abs(H - H.T).max() < 1e-15


def test_ggn_null_space_and_zero_weights(ggn_small):
    g = ggn_small
    a = wl.normal_vector(3, 52, g.d).astype(np.float64)
    shift_dir = np.outer(a, np.ones(g.C)).reshape(-1)            # adding a_i to every class logit
    assert np.abs(oracle.hvp_softmax_ggn(g.X, g.W, shift_dir)).max() < 1e-14
    # W = 0: H = (X^T X / B) kron (I/C - 11^T/C^2); its non-zero eigenvalues are eig(X^T X / B) / C
    X = g.X.astype(np.float64)
    op = lambda v: oracle.hvp_softmax_ggn(g.X, np.zeros_like(g.W), v)
    H = np.column_stack([op(e) for e in np.eye(g.n)])
    got = np.sort(np.linalg.eigvalsh(H))[::-1]
    base = np.sort(np.linalg.eigvalsh(X.T @ X / g.B))[::-1] / g.C
    expect = np.sort(np.repeat(base, g.C - 1))[::-1]
    assert np.allclose(got[: len(expect)], expect, atol=1e-12)
    assert np.abs(got[len(expect):]).max() < 1e-12


def test_ggn_lanczos_top_values_match_dense(ggn_small):
    g = ggn_small
    op = lambda v: oracle.hvp_softmax_ggn(g.X, g.W, v)
    H = np.column_stack([op(e) for e in np.eye(g.n)])
    res = oracle.lanczos(op, g.v1, 30, passes=2)
    rz = oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, 4, 0)
    ev = np.linalg.eigvalsh(H)[::-1]
    assert np.max(np.abs(rz.evals - ev[:4]) / ev[:4]) < 1e-8


# ---------------------------------------------------------------- stored values
def test_oracle_reproduces_stored_values(cfg1):
    """Guards the oracle's arithmetic against silent edits: the stored file was
    written by tests/golden/make_golden.py from the oracle alone."""
    import json
    import os
    w, res = cfg1
    with open(os.path.join(os.path.dirname(__file__), "golden", "cfg1_oracle.json")) as f:
        gold = json.load(f)
    assert res.m_eff == gold["m_eff"]
    # early entries are well conditioned; late ones amplify rounding differences between BLAS builds
    assert np.allclose(res.alpha[:20], gold["alpha"][:20], rtol=1e-9, atol=1e-9)
    assert np.allclose(res.beta[:20], gold["beta"][:20], rtol=1e-9, atol=1e-9)
    rz = oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, w.k, w.l)
    assert np.allclose(rz.evals, gold["ritz_top10"], rtol=1e-10)
    p = w.params
    w1, b1 = oracle.fosi_step(w.w0, w.grad(0), rz.V, rz.evals, np.zeros(w.n),
                              float(p.alpha), float(p.lr), float(p.momentum))
    assert np.isclose(np.linalg.norm(w1 - w.w0), gold["step_update_norm"], rtol=1e-9)
    assert np.isclose(np.linalg.norm(b1), gold["momentum_norm"], rtol=1e-9)


def test_second_pass_option_on_a_long_run():
    """The oracle's optional second Gram-Schmidt pass, pinned where it matters: a run that nearly exhausts the
    Krylov space (rank 128 + shift, 127 steps).  With it the basis is orthonormal to rounding, every Ritz value
    lies inside the spectrum and the converged ones equal planted eigenvalues; the single pass of the printed
    algorithm has lost orthogonality by then even in float64."""
    n, r, m = 900, 128, 127
    rng = np.random.default_rng(3)
    U = np.linalg.qr(rng.standard_normal((n, r)))[0]
    lam = np.concatenate([np.geomspace(40.0, 0.5, r - 10), -np.geomspace(2.0, 0.2, 10)])
    shift = 0.05
    v1 = rng.standard_normal(n)
    hv = lambda v: U @ (lam * (U.T @ v)) + shift * v
    two = oracle.lanczos(hv, v1, m, passes=2)
    assert two.m_eff == m
    Q = two.Q[:, :m]
    assert np.abs(Q.T @ Q - np.eye(m)).max() < 1e-12
    rz = oracle.ritz(two.Q, two.alpha, two.beta, two.m_eff, 12, 6)
    truth = np.sort(np.concatenate([lam + shift, [shift]]))
    assert rz.all_evals.min() >= truth[0] - 1e-9 and rz.all_evals.max() <= truth[-1] + 1e-9
    conv = rz.resid <= 1e-9 * np.abs(rz.evals)
    assert conv.sum() >= 12
    for ev in rz.evals[conv]:
        assert np.min(np.abs(truth - ev)) <= 1e-8 * max(1.0, abs(ev))
    one = oracle.lanczos(hv, v1, m, passes=1)
    Q1 = one.Q[:, : one.m_eff]
    assert np.abs(Q1.T @ Q1 - np.eye(one.m_eff)).max() > 1e-6


def test_newton_term_printed_and_simplified_forms_agree_on_an_fp32_basis():
    """Eq. 4 / Eq. 14 print the Newton term with V^T applied to the projected gradient V (V^T g~); for orthonormal V
    that is V^T g~.  The device uses the short form on a basis stored in fp32 (orthonormal to ~1e-7): the two
    forms must then agree far inside the 1e-5 bar of the update."""
    rng = np.random.default_rng(17)
    n, r = 20000, 30
    V = np.linalg.qr(rng.standard_normal((n, r)))[0].astype(np.float32).astype(np.float64)
    assert 1e-9 < np.abs(V.T @ V - np.eye(r)).max() < 1e-6            # rounded: no longer exactly orthonormal
    ev = np.concatenate([rng.uniform(1, 50, 20), -rng.uniform(0.5, 5, 10)])
    w0, g, b0, pi = (rng.standard_normal(n) for _ in range(4))
    alpha, lr, mu, sigma = 0.1, 0.01, 0.9, 5e-4
    w1, b1 = oracle.fosi_step(w0, g, V, ev, b0, alpha, lr, mu, sigma, pi=pi)
    gt = g + pi
    c = V.T @ gt                                                     # short form
    b_s = mu * b0 + gt - V @ c
    o = -lr * b_s
    w_s = w0 - alpha * (V @ (c / (ev + sigma))) + o - V @ (V.T @ o)
    assert rel_l2(w_s - w0, w1 - w0) < 1e-6 and rel_l2(b_s, b1) < 1e-6
    assert rel_l2(w_s - w0, w1 - w0) > 0.0                           # ... and they are two different computations


def test_chunked_float64_state_equals_the_oracle():
    """tests/helpers.Float64State (library float64 operations in row chunks, used by the GPU test of the largest
    workload's whole schedule, where the numpy oracle cannot hold the vectors) against the oracle itself: two outer
    iterations of Algorithm 3 with three updates each, the basis changing in between."""
    import torch
    from tests.helpers import Float64State
    rng = np.random.default_rng(23)
    n, r = 7001, 9
    w0 = rng.standard_normal(n).astype(np.float32)
    alpha, lr, mu, sigma = 0.1, 0.01, 0.9, 5e-4
    st = Float64State(torch.from_numpy(w0), chunk=1000)
    w_ref, b_ref, pi_ref = w0.astype(np.float64), np.zeros(n), np.zeros(n)
    for outer in range(2):
        V = np.linalg.qr(rng.standard_normal((n, r)))[0].astype(np.float32)
        ev = np.concatenate([rng.uniform(1, 50, 6), -rng.uniform(0.5, 5, 3)])
        Vm = torch.from_numpy(np.ascontiguousarray(V.T))
        st.begin(sigma)
        a_ref, w_ref = oracle.admm_begin(w_ref, pi_ref, sigma)
        for t in range(3):
            g = (0.03 * rng.standard_normal(n)).astype(np.float32)
            st.step(Vm, ev, torch.from_numpy(g), alpha, lr, mu, sigma)
            w_ref, b_ref = oracle.fosi_step(w_ref, g, V, ev, b_ref, alpha, lr, mu, sigma, pi=pi_ref)
        st.end(sigma)
        pi_ref = oracle.admm_end(a_ref, w_ref, pi_ref, sigma)
        assert rel_l2(st.w.numpy(), w_ref) < 1e-13 and rel_l2(st.b.numpy(), b_ref) < 1e-13
        assert rel_l2(st.pi.numpy(), pi_ref) < 1e-10 and rel_l2(st.anchor.numpy(), a_ref) < 1e-13
