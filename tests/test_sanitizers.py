"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the host code, on the CPU:
the oracle (plain C) and the library's host layer (argument checks, geometry, operand-table
planning, variant choice, the tuner's loop, the tuning cache and its file format) with
stand-ins for the HIP runtime and the kernel launchers.  GPU code is not sanitized here."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600, **kw)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout[-4000:]
    return r.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc"] + SAN + [os.path.join(ROOT, "oracle", "nm_oracle.c"),
                          os.path.join(ROOT, "tests", "sanitize", "oracle_san_main.c"),
                          "-lm", "-pthread", "-o", exe])
    assert "oracle sanitizer run: ok" in _run([exe], env=ENV)


def test_api_host_layer_under_asan_ubsan(tmp_path):
    clang = "/opt/rocm/lib/llvm/bin/clang++"
    if not os.path.exists(clang):
        clang = shutil.which("amdclang++")
    if not clang:
        pytest.skip("no HIP-aware clang++ in this image")
    exe = str(tmp_path / "api_san")
    # host pass only: no device code, no HIP runtime library -- the driver file supplies both
    _run([clang, "-x", "hip", "--cuda-host-only", "-std=c++17", "-D__HIP_PLATFORM_AMD__"] + SAN +
         ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2507_17301_amd", "csrc"),
          "-I", "/opt/rocm/include",
          os.path.join(ROOT, "paper_2507_17301_amd", "csrc", "nm_api.hip"),
          os.path.join(ROOT, "tests", "sanitize", "api_host_san.cpp"), "-o", exe])
    assert "host-layer sanitizer run: ok" in _run([exe, str(tmp_path)], env=ENV)
