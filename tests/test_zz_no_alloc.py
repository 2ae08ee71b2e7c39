"""The entry point that allocates nothing: fosi_step_noalloc (static device scratch, no context) must reproduce
fosi_step -- same kernels, same launch shapes -- on two calls in a row, the second on a smaller input, with and
without a dual variable, and must refuse more columns than its static array was sized for."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


def _case(fo, ctx, n, r_v, with_pi, seed):
    rng = np.random.default_rng(seed)
    ld = wl.padded_ld(n)
    Vh = np.linalg.qr(rng.standard_normal((n, max(r_v, 1))))[0][:, :r_v].astype(np.float32)
    V = fo.ColMajor.from_numpy(Vh, ld) if r_v > 0 else None
    ev = np.concatenate([rng.uniform(1.0, 50.0, r_v - r_v // 3), -rng.uniform(0.5, 5.0, r_v // 3)])
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    w0, g, b0 = (rng.standard_normal(n).astype(np.float32) for _ in range(3))
    pi = (0.1 * rng.standard_normal(n)).astype(np.float32) if with_pi else None
    sp = fo.StepParams(0.1, 0.01, 0.9, 5e-4, 0)
    # the existing entry point
    w_a, m_a = dev(w0), dev(b0)
    fo.fosi_step(ctx, V, r_v, ev, dev(g), dev(pi) if with_pi else None, m_a, w_a, sp)
    ctx.synchronize()
    # the one that allocates nothing; torch's allocator is watched around the call itself
    w_b, m_b, g_d = dev(w0), dev(b0), dev(g)
    pi_d = dev(pi) if with_pi else None
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    fo.fosi_step_noalloc(None, V, r_v, ev, g_d, pi_d, m_b, w_b, sp)
    after = torch.cuda.memory_stats()["allocation.all.allocated"]
    torch.cuda.synchronize()
    assert after == before
    return (w_a.cpu().numpy(), m_a.cpu().numpy()), (w_b.cpu().numpy(), m_b.cpu().numpy()), (w0, g, b0, pi, Vh, ev)


def test_noalloc_update_matches_the_context_entry_point_twice_in_a_row():
    import oracle
    import paper_2505_00982_amd as fo
    from tests.helpers import rel_l2
    ctx = fo.Context(0)
    try:
        # two calls in a row on the shared static scratch, the second smaller in rows and columns (stale partial
        # sums and coefficients of the first call lie beyond what the second one writes)
        for n, r_v, with_pi, seed in ((300_007, 40, True, 1), (70_001, 7, False, 2), (4_099, 0, True, 3)):
            (w_a, m_a), (w_b, m_b), (w0, g, b0, pi, Vh, ev) = _case(fo, ctx, n, r_v, with_pi, seed)
            assert np.array_equal(w_a, w_b) and np.array_equal(m_a, m_b), (n, r_v)
            # and both sit at the oracle's bar for the update (relative L2 error 1e-5)
            f32 = lambda x: float(np.float32(x))
            w_ref, b_ref = oracle.fosi_step(w0, g, Vh, ev, b0, f32(0.1), f32(0.01), f32(0.9), f32(5e-4), pi=pi)
            assert rel_l2(w_b, w_ref) <= 1e-5 and rel_l2(m_b, b_ref) <= 1e-5
    finally:
        ctx.close()


def test_noalloc_update_refuses_sizes_beyond_its_static_array():
    import paper_2505_00982_amd as fo
    n, r_v = 1024, 65
    V = fo.ColMajor(n, r_v)
    z = torch.zeros(n, device="cuda")
    with pytest.raises(fo.FosiError) as e:
        fo.fosi_step_noalloc(None, V, r_v, np.ones(r_v), z, None, z.clone(), z.clone(), fo.StepParams())
    assert e.value.status == -8          # FOSI_ERR_LIMIT
    with pytest.raises(fo.FosiError) as e:
        fo.fosi_step_noalloc(None, V, 3, np.array([1.0, -0.5, 2.0]), z, z.clone(), z.clone(), z.clone(),
                             fo.StepParams(sigma=0.5))
    assert e.value.status == -4          # a zero Newton divisor
