"""Host sanitizer run of the CPU oracle: oracle/gc_oracle.cpp and a driver that walks all of its
entry points are compiled with -fsanitize=address,undefined (no recovery) and executed once. Any
out-of-bounds access, signed overflow, misaligned access or leak fails the run."""
import os
import shutil
import subprocess

import pytest

from tests.conftest import ROOT


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "oracle_san")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           os.path.join(ROOT, "tests", "san", "oracle_sanitize_main.cpp"),
           os.path.join(ROOT, "oracle", "gc_oracle.cpp"), "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "asan" in (built.stderr or "").lower() and "cannot find" in built.stderr:
        pytest.skip("sanitizer runtime not installed")
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "oracle sanitizer run: ok" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr


def test_launch_constant_division_is_exact(tmp_path):
    """Host logic of the library: the multiply-shift constants that replace `pair / block` in the
    kernels (csrc/gc_fastdiv.h), compiled for the host and checked against the plain quotient on
    edge and random dividends for fixed and random divisors."""
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "fastdiv")
    built = subprocess.run([gxx, "-std=c++17", "-O2", os.path.join(ROOT, "tests", "san", "fastdiv_main.cpp"), "-o", exe],
                           capture_output=True, text=True)
    assert built.returncode == 0, built.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "0 mismatches" in run.stdout
