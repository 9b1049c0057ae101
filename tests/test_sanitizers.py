"""Sanitizer builds of everything in this repository that runs on the host (CPU only; the GPU code has its own
parity tests).

* the oracle (oracle/ciar_oracle.c) with tests/sanitize/oracle_driver.c under AddressSanitizer +
  UndefinedBehaviorSanitizer (gcc);
* the C ABI's host code (csrc/ciar_api.cpp: validation, parameter resolution, workspace carving, the look-up of the
  built-in scratch buffer) with the stand-in launchers of tests/sanitize/api_stubs.cpp, once under AddressSanitizer +
  UndefinedBehaviorSanitizer and once under ThreadSanitizer (clang).  The file is compiled as plain C++ here: the
  two HIP spellings it uses for its device array are given their host meaning on the command line.

A driver exits 0 when its expectations held; a sanitizer report aborts it."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
API = os.path.join(ROOT, "paper_2603_25463_amd", "csrc", "ciar_api.cpp")
CLANG = "/opt/rocm/llvm/bin/clang++"
AS_PLAIN_CXX = ["-x", "c++", "-D__HIP_PLATFORM_AMD__", "-D__align__(n)=__attribute__((aligned(n)))", "-DHIP_SYMBOL(x)=x",
                "-I/opt/rocm/include"]


def _run(exe, **env):
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=dict(os.environ, **env))
    assert r.returncode == 0, (r.stdout[-1500:] + r.stderr[-3000:])
    assert "0 failed expectations" in r.stdout


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_asan")
    subprocess.run(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-static-libasan", "-fno-omit-frame-pointer",
                    os.path.join(SAN, "oracle_driver.c"), "-o", exe, "-lm"], check=True)
    _run(exe, ASAN_OPTIONS="detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")


@pytest.mark.parametrize("sanitize", ["address,undefined", "thread"])
def test_c_abi_host_code_under_sanitizers(tmp_path, sanitize):
    if not os.path.exists(CLANG):
        pytest.skip("ROCm's clang++ is not installed")
    exe = str(tmp_path / "api_san")
    cmd = [CLANG, "-O1", "-g", "-std=c++17", *AS_PLAIN_CXX, f"-fsanitize={sanitize}", "-fno-omit-frame-pointer"]
    if sanitize != "thread":
        cmd.append("-fno-sanitize-recover=all")
    cmd += [API, os.path.join(SAN, "api_stubs.cpp"), os.path.join(SAN, "api_driver.cpp"), "-o", exe, "-lpthread"]
    subprocess.run(cmd, check=True)
    _run(exe, TSAN_OPTIONS="halt_on_error=1 exitcode=66", ASAN_OPTIONS="detect_leaks=1")
