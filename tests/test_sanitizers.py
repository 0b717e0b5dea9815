"""CPU-only sanitizer tier: the fp64 oracle and the host side of libvsprefill (argument validation, workspace layouts:
everything between the C ABI and the first kernel launch) built with AddressSanitizer + UndefinedBehaviorSanitizer and
run through small drivers.  The sanitizer runtimes are linked statically into the drivers; a report aborts the run."""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")


def _run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "run ok" in r.stdout, r.stdout[-2000:]


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-pthread", os.path.join(SAN, "oracle_driver.cpp"),
           os.path.join(ROOT, "oracle", "vs_oracle.cpp"), "-o", exe]
    subprocess.check_call(cmd)
    out = subprocess.run(["nm", exe], stdout=subprocess.PIPE, text=True).stdout
    assert "__asan_init" in out and "__ubsan_handle" in out
    _run(exe)


def test_host_glue_under_asan_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not installed")
    exe = str(tmp_path / "host_san")
    srcs = sorted(glob.glob(os.path.join(ROOT, "paper_2603_04460_amd", "csrc", "*.hip")))
    # sanitizer flags apply to the host pass only (each one directly after -Xarch_host); device code is built as usual
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-w",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2603_04460_amd", "csrc")] + srcs + [
           os.path.join(SAN, "host_driver.cpp"), "-o", exe]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-4000:]
    out = subprocess.run(["nm", exe], stdout=subprocess.PIPE, text=True).stdout
    assert "__asan_init" in out
    _run(exe)
