"""The CPU oracle and the host side of the C ABI under AddressSanitizer and
UndefinedBehaviorSanitizer (host code only; GPU code is not instrumented).

  oracle:  g++ -fsanitize=address,undefined  oracle/oracle.cpp tests/sanitize/oracle_driver.cpp
  ABI:     hipcc, with each -fsanitize= option directly after -Xarch_host, on csrc/api.hip,
           csrc/policy.hip and tests/sanitize/abi_driver.cpp (kernel launchers stubbed)

Each driver must print "ok" and the sanitizers must report nothing."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1",
           OMP_NUM_THREADS="4")


def _run(cmd, exe, tmp_path):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-3000:]
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=ENV, cwd=str(tmp_path))
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), (r.stdout[-2000:], r.stderr[-3000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]


def test_oracle_under_asan_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "oracle_san")
    _run([gxx, "-O1", "-g", "-std=c++17", "-fopenmp", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
          os.path.join(ROOT, "oracle", "oracle.cpp"), os.path.join(SAN, "oracle_driver.cpp"), "-o", exe], exe, tmp_path)


def test_abi_host_code_under_asan_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    exe = str(tmp_path / "abi_san")
    csrc = os.path.join(ROOT, "paper_2308_15030_amd", "csrc")
    _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
          "-I", os.path.join(ROOT, "include"), "-I", csrc,
          os.path.join(csrc, "api.hip"), os.path.join(csrc, "policy.hip"), "-x", "hip", os.path.join(SAN, "abi_driver.cpp"),
          "-o", exe], exe, tmp_path)
