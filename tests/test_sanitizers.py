"""Oracle and host code under AddressSanitizer + UBSan (CPU only; GPU code is not
instrumented: the sanitizer flags go to the host pass alone)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def test_oracle_under_asan_ubsan(tmp_path):
    exe = tmp_path / "oracle_driver"
    subprocess.run(["gcc", "-std=c11", *SAN, "-ffp-contract=off", os.path.join(ROOT, "oracle", "cdsgd_oracle.c"),
                    os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), "-o", str(exe), "-lm"], check=True)
    r = subprocess.run([str(exe)], env=ENV, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "oracle driver ok" in r.stdout


def test_library_host_code_under_asan_ubsan(tmp_path):
    """The library's host side (argument checks, plan bookkeeping up to the first HIP call, the
    trainer counter, the time model) built by hipcc with the sanitizers on the host pass only."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = tmp_path / "host_driver"
    host_san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"):
        host_san += ["-Xarch_host", f]
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           *host_san, "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "paper_2106_10796_amd", "csrc", "cdsgd.hip"),
           os.path.join(ROOT, "paper_2106_10796_amd", "csrc", "cdsgd_cost_model.cpp"),
           os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"), "-o", str(exe)]
    b = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert b.returncode == 0, b.stdout[-3000:]
    # leak detection off: the HIP runtime's own start-up allocations are not ours to judge
    env = dict(ENV, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0")
    r = subprocess.run([str(exe)], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "host driver: 0 failed checks" in r.stdout
