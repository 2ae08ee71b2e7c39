"""CPU-side checks of the shared library: it loads, exports every function the
header declares, and its host-only code (the tridiagonal eigen-solver, status
strings) is correct.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def fo():
    import paper_2505_00982_amd as fo
    if not os.path.exists(fo.library_path()):
        from paper_2505_00982_amd.build import build_library
        build_library(verbose=False)
    return fo


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fosi.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(?:fosi_status|const char\*|int32_t|size_t)\s+((?:fosi|hvp)_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_header_declares_the_boundary():
    names = declared_functions()
    for must in ("fosi_lanczos", "fosi_ritz", "fosi_step", "fosi_admm_begin", "fosi_admm_end", "hvp_planted_create",
                 "hvp_diag_create", "hvp_softmax_ggn_create", "hvp_callback_create", "hvp_apply", "hvp_destroy",
                 "fosi_ctx_create", "fosi_tridiag_eigh"):
        assert must in names


def test_library_exports_every_declared_symbol(fo):
    lib = fo.load_library()
    for name in declared_functions():
        assert hasattr(lib, name), name
    assert sorted(fo.binding.EXPORTS) == declared_functions()


def test_status_strings(fo):
    lib = fo.load_library()
    assert lib.fosi_status_string(0) == b"ok"
    assert b"layout" in lib.fosi_status_string(-2)
    assert lib.fosi_status_string(-99) == b"unknown status"
    assert lib.fosi_last_error(None) == b"null context"


@pytest.mark.parametrize("m", [1, 2, 3, 17, 61, 101, 255])
def test_tridiagonal_solver_against_lapack(fo, m):
    rng = np.random.default_rng(m)
    a = rng.standard_normal(m) * 10.0 ** rng.uniform(-2, 4, m)
    b = np.abs(rng.standard_normal(max(m - 1, 0))) * 10.0 ** rng.uniform(-3, 3, max(m - 1, 0))
    ev, Z = fo.fosi_tridiag_eigh(a, b)
    T = np.diag(a) + (np.diag(b, 1) + np.diag(b, -1) if m > 1 else 0)
    ref = np.linalg.eigvalsh(T)
    scale = max(np.abs(ref).max(), 1e-300)
    assert np.all(np.diff(ev) >= 0)
    assert np.abs(ev - ref).max() <= 1e-13 * scale
    assert np.abs(T @ Z - Z * ev).max() <= 1e-12 * scale
    assert np.abs(Z.T @ Z - np.eye(m)).max() <= 1e-12


def test_tridiagonal_solver_special_cases(fo):
    # decoupled blocks (zero off-diagonal entries) and repeated eigenvalues
    a = np.array([2.0, 2.0, 5.0, 5.0, -1.0])
    b = np.array([0.0, 0.0, 0.0, 0.0])
    ev, Z = fo.fosi_tridiag_eigh(a, b)
    assert np.allclose(ev, [-1, 2, 2, 5, 5])
    assert np.abs(Z.T @ Z - np.eye(5)).max() < 1e-14
    # the (1, -2, 1)-type matrix has the closed-form spectrum 2 - 2 cos(j pi / (m+1))
    m = 50
    ev = fo.fosi_tridiag_eigh(np.full(m, 2.0), np.full(m - 1, -1.0), vectors=False)
    j = np.arange(1, m + 1)
    assert np.abs(ev - (2 - 2 * np.cos(j * np.pi / (m + 1)))).max() < 1e-13


def test_tridiagonal_solver_on_generated_matrices(fo):
    """Property test over generated tridiagonals: sizes 1..40, entries spanning many orders of magnitude, exact
    zeros on the off-diagonal (decoupled blocks), repeated diagonal entries, negative off-diagonal entries."""
    from hypothesis import given, settings, strategies as st

    magnitudes = st.sampled_from([0.0, 1e-12, 1e-3, 1.0, 7.5, 1e4, 1e9])
    entry = st.tuples(st.sampled_from([-1.0, 1.0]), magnitudes, st.floats(0.5, 1.5)).map(lambda t: t[0] * t[1] * t[2])
    repeated = st.sampled_from([2.0, 2.0, -3.0, 0.0])

    @settings(max_examples=150, deadline=None, derandomize=True)
    @given(st.integers(1, 40).flatmap(lambda m: st.tuples(
        st.lists(st.one_of(entry, repeated), min_size=m, max_size=m),
        st.lists(entry, min_size=max(m - 1, 0), max_size=max(m - 1, 0)))))
    def check(ab):
        a, b = np.array(ab[0], dtype=np.float64), np.array(ab[1], dtype=np.float64)
        m = len(a)
        ev, Z = fo.fosi_tridiag_eigh(a, b)
        T = np.diag(a) + (np.diag(b, 1) + np.diag(b, -1) if m > 1 else 0)
        scale = max(np.abs(T).sum(axis=1).max(), 1e-300)           # infinity norm bounds the spectrum
        assert np.all(np.diff(ev) >= 0)
        assert np.abs(ev - np.linalg.eigvalsh(T)).max() <= 1e-13 * scale
        assert np.abs(T @ Z - Z * ev).max() <= 1e-12 * scale
        assert np.abs(Z.T @ Z - np.eye(m)).max() <= 1e-12

    check()


def test_tridiagonal_solver_rejects_bad_input(fo):
    lib = fo.load_library()
    ev = np.zeros(3)
    dp = C.POINTER(C.c_double)
    a = np.array([1.0, np.nan, 2.0])
    b = np.array([1.0, 1.0, 0.0])
    assert lib.fosi_tridiag_eigh(3, a.ctypes.data_as(dp), b.ctypes.data_as(dp), ev.ctypes.data_as(dp), None) == -4
    assert lib.fosi_tridiag_eigh(0, a.ctypes.data_as(dp), b.ctypes.data_as(dp), ev.ctypes.data_as(dp), None) == -1
    assert lib.fosi_tridiag_eigh(3, None, b.ctypes.data_as(dp), ev.ctypes.data_as(dp), None) == -1


def test_null_context_is_rejected_without_touching_a_gpu(fo):
    lib = fo.load_library()
    assert lib.fosi_ctx_synchronize(None) == -1
    assert lib.fosi_ctx_destroy(None) == -1
    assert lib.hvp_apply(None, None, None) == -1
    assert lib.fosi_profile_enable(None, 1) == -1
    assert lib.fosi_admm_begin(None, 10, 0.1, None, None, None) == -1
    assert lib.fosi_lanczos_second_passes(None, None) == -1
    assert lib.fosi_lanczos_end(None, None, None, None) == -1


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr


def test_lanczos_length_rule(fo):
    # m = max{4 (k + l), 2 ln n}
    assert fo.fosi_lanczos_steps(4096, 10, 0) == 40
    assert fo.fosi_lanczos_steps(25_600_000, 20, 10) == 120
    assert fo.fosi_lanczos_steps(10 ** 9, 1, 0) == int(np.ceil(2 * np.log(1e9)))      # the size term wins: 42
    assert fo.fosi_lanczos_steps(0, 1, 0) == 0 and fo.fosi_lanczos_steps(10, 0, 0) == 0


def test_bf16_rounding_of_the_generator_matches_torch():
    """The second softmax-GGN workload rounds its data matrix to bf16 on the host; the rounding (nearest,
    ties to even) is checked against torch's conversion, including ties and values next to them."""
    import torch
    import workloads as wl
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 3.0,
                        np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 3.0e-39, 65280.0, 1.0 + 2.0 ** -9],
                                 dtype=np.float32)])
    ties = (np.arange(1, 400, dtype=np.float32) * np.float32(2.0 ** -8)) + np.float32(1.0)      # half-way points of [1, 2)
    x = np.concatenate([x, ties, np.nextafter(ties, np.float32(0)), np.nextafter(ties, np.float32(4))])
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(wl.generators.round_to_bf16(x), ref)


def test_header_is_plain_c_and_links_from_c(fo, tmp_path):
    """The boundary is a C ABI: the header compiles as C99 (pedantic, no C++), and a C program links against the
    library and calls a host-only entry point."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_header.c"
    src.write_text('#include "fosi.h"\n'
                   "int main(void) {\n"
                   "    fosi_lanczos_opts o = {0};\n"
                   "    double a[3] = {2.0, 2.0, 2.0}, b[2] = {-1.0, -1.0}, ev[3];\n"
                   "    (void)o;\n"
                   "    if (fosi_lanczos_steps(4096, 10, 0) != 40) return 1;\n"
                   "    if (fosi_tridiag_eigh(3, a, b, ev, 0) != FOSI_OK) return 2;\n"
                   "    return (ev[0] < ev[1] && ev[1] < ev[2] && ev[1] > 1.999999 && ev[1] < 2.000001) ? 0 : 3;\n"
                   "}\n")
    libdir = os.path.dirname(fo.library_path())
    exe = tmp_path / "use_header"
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                        str(src), "-o", str(exe), "-L", libdir, "-lfosi_hip", f"-Wl,-rpath,{libdir}"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, (r.returncode, r.stderr)


def test_workspace_query_is_host_only_and_size_independent(fo):
    lib = fo.load_library()
    w = lib.fosi_workspace_bytes(25_600_000, 80, 30)
    assert 8 << 20 < w < 16 << 20
    assert lib.fosi_workspace_bytes(4096, 1, 0) == w
    assert lib.fosi_workspace_bytes(0, 80, 30) == 0 and lib.fosi_workspace_bytes(4096, 256, 0) == 0
