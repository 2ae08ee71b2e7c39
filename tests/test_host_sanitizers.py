"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only; device code is never instrumented).

  * the tridiagonal eigen-solver, compiled on its own with g++ and driven by tests/host_harness/tridiag_harness.cpp;
  * the whole library built with hipcc with the sanitizers on the host pass only, driven through the argument-checking
    paths of every exported function by tests/host_harness/argcheck_harness.cpp (null contexts, bad sizes, limits;
    nothing reaches a kernel launch).
A sanitizer report makes the harness exit non-zero."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_00982_amd", "csrc")
HARNESS = os.path.join(ROOT, "tests", "host_harness")
SAN_ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def test_tridiagonal_solver_under_asan_and_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "tridiag_harness")
    subprocess.run([gxx, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    os.path.join(CSRC, "tridiag_eigh.cpp"), os.path.join(HARNESS, "tridiag_harness.cpp"), "-o", exe],
                   check=True)
    out = subprocess.run([exe], env=SAN_ENV, capture_output=True, text=True, timeout=600)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "tridiag harness ok" in out.stdout


def test_argument_checks_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    from paper_2505_00982_amd.build import SOURCES
    lib = str(tmp_path / "libfosi_hip_san.so")
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined"]
    subprocess.run([hipcc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", *host_san,
                    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-result",
                    "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", lib]
                   + [os.path.join(CSRC, s) for s in SOURCES], check=True, capture_output=True)
    exe = str(tmp_path / "argcheck_harness")
    subprocess.run([hipcc, "-O1", "-g", "-std=c++17", "-x", "c++", *host_san, "-I", os.path.join(ROOT, "include"),
                    os.path.join(HARNESS, "argcheck_harness.cpp"), "-x", "none", lib, "-Wl,-rpath," + str(tmp_path), "-o", exe],
                   check=True, capture_output=True)
    out = subprocess.run([exe], env=SAN_ENV, capture_output=True, text=True, timeout=600)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "argcheck harness ok" in out.stdout
