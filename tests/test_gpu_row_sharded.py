"""Row-sharded Lanczos (Algorithm 2) emulated on one GPU: the per-block partial
sums, added in rank order, must reproduce the single-device recurrence, and both
must agree with the CPU oracle's emulation of the same algorithm."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from oracle.lanczos import lanczos_row_sharded
from tests.helpers import sin_principal_angles

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


def run(fo, ctx, w, op, m, shards, mode):
    ld = wl.padded_ld(w.n)
    Q = fo.ColMajor(w.n, m + 1, ld)
    Q.col(0).copy_(dev(w.v1))
    if shards == 0:
        a, b, me = fo.fosi_lanczos(ctx, op, Q, m, reorth_mode=mode)
    else:
        a, b, me = fo.fosi_lanczos_row_sharded(ctx, op, Q, m, shards, reorth_mode=mode)
    ctx.synchronize()
    return a, b, me, Q


# 70001 rows: block boundaries at multiples of 64, a ragged last block with n mod 4 = 1;
# 8 blocks of 8768 rows; 64 requested blocks become 61 of 1152 rows (empty ones are dropped)
@pytest.mark.parametrize("mode", [1, 2, 3])
@pytest.mark.parametrize("shards", [1, 3, 8, 64])
def test_sharded_recurrence_matches_single_device(fo, ctx, shards, mode):
    w = wl.planted_workload(2, n=70001)
    m = 20
    U = fo.ColMajor.from_numpy(w.U, wl.padded_ld(w.n))
    op = ctx.hvp_planted(U, dev(w.lam), float(w.shift))
    a0, b0, me0, Q0 = run(fo, ctx, w, op, m, 0, mode)
    a1, b1, me1, Q1 = run(fo, ctx, w, op, m, shards, mode)
    assert me0 == me1 == m
    scale = np.abs(w.lam).max()
    # same arithmetic, different summation order of fp64 partial sums; a single pass amplifies the
    # rounding differences of the stored fp32 vectors from step to step, hence the looser bound there
    tol = 1e-9 if mode != 1 else 1e-5
    nchk = m if mode != 1 else 8
    assert np.max(np.abs(a0[:nchk] - a1[:nchk])) <= tol * scale
    assert np.max(np.abs(b0[:nchk] - b1[:nchk])) <= tol * scale
    if mode != 1:
        A, B = Q0.to_numpy(m).astype(np.float64), Q1.to_numpy(m).astype(np.float64)
        assert np.max(np.abs(A - B)) <= 1e-6          # fp32 columns: identical up to a last-bit flip now and then
    op.close()


def test_sharded_against_oracle_emulation(fo, ctx):
    w = wl.planted_workload(2, n=50000)
    m, k, l, shards = 30, 4, 2, 5
    U = fo.ColMajor.from_numpy(w.U, wl.padded_ld(w.n))
    op = ctx.hvp_planted(U, dev(w.lam), float(w.shift))
    a, b, me, Q = run(fo, ctx, w, op, m, shards, 0)
    hv = lambda v: oracle.hvp_planted(w.U, w.lam, float(w.shift), v)
    res = lanczos_row_sharded(hv, w.v1, m, shards)
    assert me == res.m_eff == m
    V = fo.ColMajor(w.n, k + l, wl.padded_ld(w.n))
    evals, _ = fo.fosi_ritz(ctx, Q, me, a, b, k, l, V)
    ctx.synchronize()
    rz = oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, k, l)
    conv = rz.resid <= 1e-6 * np.abs(rz.evals)
    assert conv.sum() >= 3
    assert np.max(np.abs(evals - rz.evals)[conv] / np.abs(rz.evals)[conv]) <= 1e-4
    Vg = V.to_numpy().astype(np.float64)
    idx = np.where(conv)[0]
    assert sin_principal_angles(rz.V[:, idx], Vg[:, idx]).max() < 1e-3
    op.close()


def test_sharded_with_whole_vector_operator(fo, ctx):
    """An operator that needs the whole vector (here the diagonal one) is applied unsharded; the
    Gram-Schmidt sums are still taken block by block."""
    n, m = 5000, 25
    d = (np.linspace(-2.0, 6.0, n) + 0.3 * np.sin(np.arange(n))).astype(np.float32)
    v1 = wl.normal_vector(1, 77, n)
    op = ctx.hvp_diag(dev(d))
    out = []
    for shards in (0, 4):
        Q = fo.ColMajor(n, m + 1)
        Q.col(0).copy_(dev(v1))
        if shards:
            a, b, me = fo.fosi_lanczos_row_sharded(ctx, op, Q, m, shards)
        else:
            a, b, me = fo.fosi_lanczos(ctx, op, Q, m)
        ctx.synchronize()
        assert me == m
        out.append((a, b))
    assert np.max(np.abs(out[0][0] - out[1][0])) <= 1e-9 * 6.0
    assert np.max(np.abs(out[0][1] - out[1][1])) <= 1e-9 * 6.0
    op.close()


def test_sharded_argument_errors(fo, ctx):
    n = 1000
    op = ctx.hvp_diag(dev(np.ones(n)))
    Q = fo.ColMajor(n, 5)
    Q.col(0).fill_(1.0)
    with pytest.raises(fo.FosiError):
        fo.fosi_lanczos_row_sharded(ctx, op, Q, 4, 0)
    with pytest.raises(fo.FosiError):
        fo.fosi_lanczos_row_sharded(ctx, op, Q, 4, 65)
    with pytest.raises(fo.FosiError, match="selective"):
        fo.fosi_lanczos_row_sharded(ctx, op, Q, 4, 2, reorth_mode=fo.REORTH_SELECTIVE)
    op.close()
