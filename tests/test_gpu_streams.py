"""Independent parameter blocks on separate streams: one context per stream, driven from host threads or, through
the begin / end halves of the Lanczos call, from one thread.  The contexts share nothing (each owns its scratch), so
concurrent runs must give exactly the numbers of a run alone."""
import threading

import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


def make_blocks(fo):
    sizes = [(30011, 16), (65536, 20), (12345, 12), (50000, 18)]
    blocks = []
    for i, (n, m) in enumerate(sizes):
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            w = wl.planted_workload(2, n=n)
            ld = wl.padded_ld(n)
            ctx = fo.Context(0, stream=stream)
            U = fo.ColMajor.from_numpy(w.U, ld)
            lam = torch.from_numpy(w.lam).cuda()
            op = ctx.hvp_planted(U, lam, float(w.shift))
            Q = fo.ColMajor(n, m + 1, ld)
            V = fo.ColMajor(n, 4, ld)
            v1 = torch.from_numpy(w.v1).cuda()
        stream.synchronize()
        blocks.append(dict(stream=stream, ctx=ctx, op=op, Q=Q, V=V, v1=v1, m=m, n=n, keep=(U, lam)))
    return blocks


def test_concurrent_contexts_reproduce_sequential_results():
    import paper_2505_00982_amd as fo
    blocks = make_blocks(fo)

    def curvature(b, out):
        with torch.cuda.stream(b["stream"]):
            for _ in range(3):
                b["Q"].col(0).copy_(b["v1"])
                a, be, me = fo.fosi_lanczos(b["ctx"], b["op"], b["Q"], b["m"])
                ev, _ = fo.fosi_ritz(b["ctx"], b["Q"], me, a, be, 3, 1, b["V"])
            b["ctx"].synchronize()
            out.append((a, be, me, ev, b["V"].buf.clone()))

    alone = []
    for b in blocks:
        res = []
        curvature(b, res)
        alone.append(res[0])
    together = [[] for _ in blocks]
    threads = [threading.Thread(target=curvature, args=(b, together[i])) for i, b in enumerate(blocks)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    for ref, got in zip(alone, together):
        assert len(got) == 1
        g = got[0]
        assert g[2] == ref[2]
        assert np.array_equal(g[0], ref[0]) and np.array_equal(g[1], ref[1]) and np.array_equal(g[3], ref[3])
        assert torch.equal(g[4], ref[4])
    for b in blocks:
        b["op"].close()
        b["ctx"].close()


def test_begin_end_halves_from_one_thread():
    """fosi_lanczos_begin on every block first (nothing waits for the GPU), then fosi_lanczos_end on each: same bits
    as the blocking call, and the misuse cases are rejected."""
    import paper_2505_00982_amd as fo
    blocks = make_blocks(fo)
    ref = []
    for b in blocks:
        with torch.cuda.stream(b["stream"]):
            b["Q"].col(0).copy_(b["v1"])
            a, be, me = fo.fosi_lanczos(b["ctx"], b["op"], b["Q"], b["m"])
            ref.append((a, be, me, b["Q"].buf.clone()))
    for rep in range(2):
        for b in blocks:
            with torch.cuda.stream(b["stream"]):
                b["Q"].col(0).copy_(b["v1"])
                fo.fosi_lanczos_begin(b["ctx"], b["op"], b["Q"], b["m"])
        with pytest.raises(fo.FosiError) as e:                       # a second run on a context that has one pending
            fo.fosi_lanczos_begin(blocks[0]["ctx"], blocks[0]["op"], blocks[0]["Q"], blocks[0]["m"])
        assert e.value.status == -1
        for b, r in zip(reversed(blocks), reversed(ref)):            # collected in another order than started
            a, be, me = fo.fosi_lanczos_end(b["ctx"], b["m"])
            assert me == r[2] and np.array_equal(a, r[0]) and np.array_equal(be, r[1])
            b["ctx"].synchronize()
            assert torch.equal(b["Q"].buf, r[3])
    with pytest.raises(fo.FosiError) as e:                           # nothing pending
        fo.fosi_lanczos_end(blocks[0]["ctx"], blocks[0]["m"])
    assert e.value.status == -1
    for b in blocks:
        b["op"].close()
        b["ctx"].close()
