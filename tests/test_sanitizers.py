"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

Two small native drivers are built with -fsanitize=address,undefined and run as child
processes: the C oracle over every n up to 64, and the argument-validation layer of the C ABI
(built for the host only, with the launchers replaced by stubs).  Any out-of-bounds access,
use after free, leak, signed overflow or misaligned access makes the sanitizer print a report
and the process exit non-zero."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
SAN_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="abort_on_error=0:detect_leaks=1:halt_on_error=1",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")


def _run(exe):
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=600)
    report = r.stdout[-2000:] + r.stderr[-6000:]
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, report
    assert r.returncode == 0, report
    return r.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    cmd = ["gcc", "-std=c99", "-fopenmp", "-ffp-contract=off"] + SAN_FLAGS + [
        "-o", exe, os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "jacobi.c"), "-lm"]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stderr[-4000:]
    assert "oracle sanitizer driver OK" in _run(exe)


def test_argument_validation_layer_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "api_driver")
    csrc = os.path.join(ROOT, "paper_2207_04228_amd", "csrc")
    host_flags = []
    for f in SAN_FLAGS:                       # hipcc: sanitizer flags go to the host compilation only
        host_flags += ["-Xarch_host", f]
    cmd = [hipcc, "--cuda-host-only", "-std=c++17", "-x", "hip"] + host_flags + [
        "-I" + os.path.join(ROOT, "include"), "-I" + csrc,
        os.path.join(csrc, "bed_api.hip"), os.path.join(SAN, "api_stubs.cpp"), os.path.join(SAN, "api_driver.cpp"),
        "-o", exe]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stderr[-4000:]
    assert "api sanitizer driver OK" in _run(exe)
