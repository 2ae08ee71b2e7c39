"""The memory-only sweep that bench.py uses as a yardstick (fosi_traffic_model) moves exactly the columns it
claims: every written column equals (w + 1) * (sum of the read columns), accumulated in column order in fp32."""
import numpy as np
import pytest
import torch

import workloads as wl

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


def _expected(A, cols_in, cols_out):
    s = np.zeros(A.shape[0], dtype=np.float32)
    for j in range(cols_in):
        s = (s + A[:, j]).astype(np.float32)
    return np.stack([(np.float32(w + 1) * s).astype(np.float32) for w in range(cols_out)], axis=1)


@pytest.mark.parametrize("n,cols_in,cols_out", [(4 * (4 * 1024 + 37), 11, 3), (8, 1, 1), (4 * 70001, 9, 2),
                                                (4 * 2048, 0, 2), (9_000_000 // 4 * 4 + 4, 5, 1)])
def test_traffic_model_moves_the_columns_it_claims(fo, ctx, n, cols_in, cols_out):
    rng = np.random.default_rng(n % 1000 + cols_in)
    Ah = rng.standard_normal((n, max(cols_in, 1))).astype(np.float32)
    A = fo.ColMajor.from_numpy(Ah, wl.padded_ld(n))
    B = fo.ColMajor(n, cols_out + 1, wl.padded_ld(n))
    B.buf.fill_(-7.0)
    fo.fosi_traffic_model(ctx, A if cols_in else None, cols_in, B, cols_out, n)
    ctx.synchronize()
    got = B.to_numpy()
    np.testing.assert_array_equal(got[:, :cols_out], _expected(Ah, cols_in, cols_out))
    assert (got[:, cols_out] == -7.0).all()                      # the column behind the last one is untouched
    pad = B.buf[: cols_out * B.ld].reshape(cols_out, B.ld)[:, n:]
    assert (pad == -7.0).all()                                   # and so is the padding between columns


def test_traffic_model_read_only_and_bad_arguments(fo, ctx):
    n = 4 * 5000
    A = fo.ColMajor.from_numpy(np.ones((n, 4), dtype=np.float32), wl.padded_ld(n))
    fo.fosi_traffic_model(ctx, A, 4, None, 0, n)                 # nothing to write: must not touch a null B
    ctx.synchronize()
    with pytest.raises(fo.FosiError):
        fo.fosi_traffic_model(ctx, A, 4, None, 0, n + 2)         # n not a multiple of 4
    with pytest.raises(fo.FosiError):
        fo.fosi_traffic_model(ctx, None, 0, None, 0, n)          # no columns at all
    with pytest.raises(fo.FosiError):
        fo.fosi_traffic_model(ctx, None, 3, None, 0, n)          # columns to read but no matrix
