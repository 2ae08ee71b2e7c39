"""HIP-graph replay of a Lanczos run: every replay must equal the eagerly launched run bit for bit, with
other work of the same program and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fo():
    import paper_2505_00982_amd as fo
    return fo


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def lanczos(fo, ctx, op, w, Q, m, graph_mode, mode=0):
    Q.col(0).copy_(dev(w.v1))
    a, b, me = fo.fosi_lanczos(ctx, op, Q, m, reorth_mode=mode, graph_mode=graph_mode)
    ctx.synchronize()
    return a, b, me, Q.buf.clone()


# the second run breaks down at step 33/34; the third uses the scheme whose second pass is switched on the device
@pytest.mark.parametrize("cfg_id,n,m,mode", [(2, 70001, 24, 0), (1, None, 40, 0), (1, None, 40, 4)])
def test_graph_replays_equal_eager(fo, cfg_id, n, m, mode):
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ctx = fo.Context(0, stream=stream)
        w = wl.planted_workload(cfg_id, n=n)
        ld = wl.padded_ld(w.n)
        U = fo.ColMajor.from_numpy(w.U, ld)
        op = ctx.hvp_planted(U, dev(w.lam), float(w.shift))
        Q = fo.ColMajor(w.n, m + 1, ld)
        ref = lanczos(fo, ctx, op, w, Q, m, fo.GRAPH_OFF, mode)
        assert ctx.graph_stats() == (0, 0)
        V = fo.ColMajor(w.n, 4, ld)
        scratch, out = torch.zeros(w.n, device="cuda"), torch.zeros(w.n, device="cuda")
        for rep in range(4):
            got = lanczos(fo, ctx, op, w, Q, m, fo.GRAPH_ON, mode)
            assert got[2] == ref[2]
            assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
            assert torch.equal(got[3], ref[3])
            # eager work of the same context between the replays: operator, Ritz vectors, an update, torch kernels
            op.apply(Q.col(1), out)
            evals, _ = fo.fosi_ritz(ctx, Q, got[2], got[0], got[1], 3, 1, V)
            fo.fosi_step(ctx, V, 4, evals, out, None, scratch, torch.zeros(w.n, device="cuda"),
                         fo.StepParams(0.1, 0.01, 0.9, 5e-4, 1))
            scratch.add_(1.0)
            torch.cuda.synchronize()
        assert ctx.graph_stats() == (1, 4)
        # another basis buffer: captured again, same numbers
        Q2 = fo.ColMajor(w.n, m + 1, ld)
        got = lanczos(fo, ctx, op, w, Q2, m, fo.GRAPH_ON, mode)
        assert np.array_equal(got[0], ref[0]) and torch.equal(got[3], ref[3])
        assert ctx.graph_stats() == (2, 5)
        # an eager run afterwards still agrees and leaves the counters alone
        got = lanczos(fo, ctx, op, w, Q2, m, fo.GRAPH_OFF, mode)
        assert ctx.graph_stats() == (2, 5) and torch.equal(got[3], ref[3])
        op.close()
        ctx.close()


def test_graph_request_on_null_stream_runs_eagerly(fo):
    ctx = fo.Context(0)                       # torch's default stream: cannot be captured
    w = wl.planted_workload(2, n=20000)
    ld = wl.padded_ld(w.n)
    U = fo.ColMajor.from_numpy(w.U, ld)
    op = ctx.hvp_planted(U, dev(w.lam), float(w.shift))
    Q = fo.ColMajor(w.n, 13, ld)
    a = lanczos(fo, ctx, op, w, Q, 12, fo.GRAPH_OFF)
    b = lanczos(fo, ctx, op, w, Q, 12, fo.GRAPH_ON)
    assert np.array_equal(a[0], b[0]) and torch.equal(a[3], b[3])
    assert ctx.graph_stats()[1] == 0
    op.close()
    ctx.close()


def test_graph_with_ggn_operator(fo):
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ctx = fo.Context(0, stream=stream)
        g = wl.ggn_workload(B=96, d=80, C=24, m=16, k=4)
        X, W = torch.from_numpy(g.X).cuda(), torch.from_numpy(g.W).cuda()
        op = ctx.hvp_softmax_ggn(X, W)
        Q = fo.ColMajor(g.n, g.m + 1, wl.padded_ld(g.n))
        res = []
        for gm in (fo.GRAPH_OFF, fo.GRAPH_ON, fo.GRAPH_ON):
            Q.col(0).copy_(torch.from_numpy(g.v1).cuda())
            a, b, me = fo.fosi_lanczos(ctx, op, Q, g.m, graph_mode=gm)
            ctx.synchronize()
            res.append((a, b, me, Q.buf.clone()))
        for r in res[1:]:
            assert r[2] == res[0][2] and np.array_equal(r[0], res[0][0]) and torch.equal(r[3], res[0][3])
        assert ctx.graph_stats() == (1, 2)
        op.close()
        ctx.close()
