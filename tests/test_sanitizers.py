"""AddressSanitizer + UndefinedBehaviorSanitizer legs, on the CPU.

  * the oracle: oracle/lbfgsb_oracle.c is compiled into tests/sanitizer/oracle_driver.c with gcc
    -fsanitize=address,undefined and driven through every entry point (all objective kinds, both storage types, the
    augmented Lagrangian algorithm, the marginal constraints, an exhausted line search);
  * the library's host side: the HIP sources are compiled with the HOST pass instrumented into
    tests/sanitizer/boundary_driver.cpp, which makes the calls the library refuses or answers before any device work
    (argument validation, workspace sizing, error strings).  No GPU is needed; device code is not instrumented.

A memory error or undefined behaviour aborts the driver (non-zero exit); so does a failed check."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitizer")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _run(exe):
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=ENV)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "all checks passed" in r.stdout
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-static-libasan", "-mfma", "-ffp-contract=off", "-Wall", "-Wextra",
                    os.path.join(SAN, "oracle_driver.c"), "-lm", "-o", exe], check=True)
    _run(exe)


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc to compile the library's sources")
def test_library_boundary_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    from paper_2203_16340_amd import build as hip_build
    exe = str(tmp_path / "boundary_san")
    srcs = [os.path.join(hip_build.CSRC, s) for s in hip_build.SOURCES]
    cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-gpu-rdc",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-gpu-sanitize",
           "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option", "-Wno-option-ignored", "-Wno-pass-failed",
           "-I", os.path.join(ROOT, "include"), "-x", "hip", *srcs, os.path.join(SAN, "boundary_driver.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, timeout=900)
    _run(exe)
