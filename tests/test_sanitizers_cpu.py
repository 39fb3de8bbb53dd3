"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer, CPU only: the fp64 checker on small inputs, and
the library's argument validation (every entry point, with pointers that are never dereferenced)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)


def test_checker_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-omit-frame-pointer", "-o", exe, os.path.join(SAN, "oracle_driver.c"),
           os.path.join(ROOT, "oracle", "slimspec_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    out = subprocess.run([exe], capture_output=True, text=True, env=dict(ENV, OMP_NUM_THREADS="4"))
    assert out.returncode == 0, out.stderr[-3000:]
    assert "status 0" in out.stdout and "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr, out.stderr[-3000:]


def test_boundary_validation_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not available")
    from paper_2605_10453_amd import build as build_mod
    exe = str(tmp_path / "boundary_san")
    flags = [f for f in build_mod.HIPCC_FLAGS if f not in ("-shared", "-O3")]
    cmd = [hipcc, *flags, "-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-omit-frame-pointer", "-o", exe, os.path.join(SAN, "boundary_driver.cpp"), *build_mod.sources()]
    subprocess.run(cmd, check=True, capture_output=True)
    out = subprocess.run([exe], capture_output=True, text=True, env=ENV)
    assert out.returncode == 0, (out.stdout[-500:], out.stderr[-3000:])
    assert "checksum" in out.stdout and "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr, out.stderr[-3000:]
