"""CPU sanitizer legs: the oracle, and the host side of the C ABI, built with AddressSanitizer and UBSan and run on
small inputs.  No GPU: the host driver only takes paths that return before anything is enqueued, and the kernel
launchers are replaced by stand-ins (tests/sanitize/host_stubs.cpp)."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _run(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    noise = "is not a recognized feature for this target"
    out = "\n".join(l for l in res.stdout.splitlines() if noise not in l)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{out}"
    return out


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
          os.path.join(ROOT, "oracle", "treekv_oracle.cpp"), os.path.join(SAN, "oracle_driver.cpp"), "-o", exe])
    assert "oracle clean" in _run([exe], env=ENV)


def test_host_side_of_the_abi_under_asan_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "host_san")
    csrc = os.path.join(ROOT, "paper_2501_04987_amd", "csrc")
    _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
          "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
          "-Xarch_host", "-fno-sanitize-recover=undefined",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
          "-I", os.path.join(ROOT, "include"), "-I", csrc,
          os.path.join(csrc, "treekv_host.hip"), "-x", "hip", os.path.join(SAN, "host_stubs.cpp"),
          os.path.join(SAN, "host_driver.cpp"), "-o", exe])
    assert "host paths clean" in _run([exe], env=ENV)
