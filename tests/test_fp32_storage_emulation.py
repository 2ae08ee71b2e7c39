"""What does keeping the Krylov basis in fp32 cost?  (CPU only.)

The device path stores the operator's output and every Lanczos vector as fp32 and does all arithmetic in wide
accumulators.  The oracle can do exactly that (`storage=numpy.float32`), so the deviations of the two largest
workloads from the float64 run can be split into what ANY implementation with fp32 vectors shows and what would be
a kernel's own loss.  The planted problem is carried by an embedding of its (r+1)-dimensional restriction into 2^16
rows: the restriction (planted spectrum, r, shift, start-vector statistics of the full-size block, Lanczos length,
k, l) is the full-size workload's, only the number of rows that share the rounding noise is smaller.

Findings pinned here (the GPU tests at full size bound the HIP path by twice these per-pair figures):
  * resolved Ritz pairs keep the stated tolerances (1e-4 relative value, 1e-3 rad);
  * the part of a Ritz vector that lies outside span([U, v1]) -- rounding noise in the (n - r)-dimensional
    eigenspace of the shift, which the recurrence amplifies along the least converged pairs -- is a deterministic
    function of the small problem: two different embeddings agree on its norm per pair;
  * n = 25.6 M workload: that part reaches ~1e-3 for the last bottom pair while the in-span angles stay far
    below 1e-3 rad; n = 125 M workload (||H|| = 1e5, m = 100): the two unresolved bottom pairs move by more than
    1e-3 rad in any fp32-storage run, in-span part included.
"""
import numpy as np
import pytest

import workloads as wl
from tests.helpers import (reduced_problem, reduced_ritz_coefficients, reduced_tridiagonal_from_gram,
                           storage_emulation, synthetic_gram)


def _setup(cfg_id):
    c = wl.CONFIGS[cfg_id]
    lam = wl.planted_spectrum(cfg_id).astype(np.float64)
    shift = float(np.float32(c["shift"]))
    G = synthetic_gram(c["r"], c["n"], seed=cfg_id)
    return c, lam, shift, G


@pytest.fixture(scope="module", params=[4, 5])
def emu(request):
    c, lam, shift, G = _setup(request.param)
    runs = [storage_emulation(G, lam, shift, c["m"], c["k"], c["l"], n_rows=1 << 16, seed=s) for s in (0, 1)]
    return request.param, c, lam, shift, G, runs


def test_float64_run_of_the_embedding_matches_the_householder_route(emu):
    """The frame itself: the float64 run on the embedded problem reproduces the tridiagonal and the Ritz values that
    LAPACK's Householder reduction of the small restricted matrix gives (an independent route)."""
    cfg_id, c, lam, shift, G, runs = emu
    m, k, l = c["m"], c["k"], c["l"]
    a_ref, b_ref = reduced_tridiagonal_from_gram(G, lam, shift)
    scale = np.abs(lam).max()
    e = runs[0]
    assert np.max(np.abs(e["alpha"] - a_ref[:m])) < 1e-8 * scale
    assert np.max(np.abs(e["beta"][: m - 1] - b_ref[: m - 1])) < 1e-8 * scale
    ev_ref, _, resid_ref, _ = reduced_ritz_coefficients(G, lam, shift, m, k, l)
    assert np.max(np.abs(e["evals"] - ev_ref)) < 1e-8 * scale
    assert np.allclose(e["resid"], resid_ref, rtol=1e-3, atol=1e-7 * scale)


def test_fp32_storage_keeps_the_stated_tolerances_on_resolved_pairs(emu):
    cfg_id, c, lam, shift, G, runs = emu
    k = c["k"]
    for e in runs:
        assert e["qtq"] < 1e-6                                      # two passes keep the fp32 basis orthonormal
        resolved = e["resid"] <= 1e-2 * np.abs(e["evals"])
        assert resolved[:k].all() and resolved.sum() > k
        assert np.max(e["value_abs_err"][resolved] / np.abs(e["evals"][resolved])) <= 1e-4
        assert np.max(np.hypot(e["out_norm"], e["in_span_leave"])[resolved]) < 1e-3
        assert e["total_sin"]["top"] < 1e-5


def test_out_of_span_part_is_a_property_of_the_problem_not_of_the_rounding_realisation(emu):
    cfg_id, c, lam, shift, G, runs = emu
    a, b = runs[0]["out_norm"], runs[1]["out_norm"]
    big = np.maximum(a, b) > 1e-5
    assert big.any()
    assert np.all(np.abs(a[big] - b[big]) <= 0.1 * np.maximum(a, b)[big])
    # ... and it is what the whole-vector angle of the bottom block consists of
    for e in runs:
        assert abs(e["total_sin"]["bottom"] - np.hypot(e["out_norm"], e["in_span_leave"]).max()) \
            <= 0.5 * e["total_sin"]["bottom"]


def test_workload4_deviation_lies_outside_the_span(emu):
    cfg_id, c, lam, shift, G, runs = emu
    if cfg_id != 4:
        pytest.skip("n = 25.6 M workload only")
    for e in runs:
        assert 1e-4 < e["total_sin"]["bottom"] < 1e-2           # what the GPU shows at full size: a few 1e-3
        assert e["in_span_sin"]["bottom"] < 1e-4                # the unique part agrees far below 1e-3 rad
        worst = int(np.argmax(e["out_norm"]))
        assert worst >= c["k"] and e["resid"][worst] > 1e-2 * abs(e["evals"][worst])   # an unresolved bottom pair


def test_workload5_unresolved_pairs_cannot_meet_one_milliradian_in_fp32_storage(emu):
    cfg_id, c, lam, shift, G, runs = emu
    if cfg_id != 5:
        pytest.skip("n = 125 M workload only")
    for e in runs:
        unresolved = e["resid"] > 1e-2 * np.abs(e["evals"])
        assert 1 <= unresolved.sum() <= 4
        assert e["total_sin"]["bottom"] > 1e-3 and e["in_span_sin"]["bottom"] > 1e-3
        moved = np.hypot(e["out_norm"], e["in_span_leave"]) > 1e-3
        assert np.all(unresolved[moved])                         # only unresolved pairs move that far
    # the late entries of the tridiagonal differ from the float64 run by far more than the early ones, in both
    # realisations alike (second-order effect of the amplified out-of-span components)
    d0, d1 = runs[0]["dT"], runs[1]["dT"]
    assert d0[-1] > 1e-3 and abs(d0[-1] - d1[-1]) <= 0.2 * d0[-1]
