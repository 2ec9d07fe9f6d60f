"""The host code of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU): builds
the library a second time with its host side instrumented, builds tests/abi_host_check.c the same way,
and runs it.  The exerciser makes a few hundred plan and entry-point calls, among them every error
path; each returns before a launch.  A sanitizer report aborts the program and fails the test."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/llvm/bin/clang"


@pytest.mark.skipif(not os.path.exists(CLANG), reason="the ROCm clang is not installed")
def test_host_logic_under_asan_and_ubsan(tmp_path):
    from paper_2410_20926_amd import build
    lib = build.build_sanitized(verbose=False)
    exe = str(tmp_path / "abi_host_check")
    subprocess.run([CLANG, "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                    "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "abi_host_check.c"), lib,
                    "-Wl,-rpath," + os.path.dirname(lib), "-Wl,-rpath,/opt/rocm/lib", "-o", exe], check=True)
    env = dict(os.environ)
    # leak checking would walk the HIP runtime's own start-up allocations; link order is checked against the preloaded harness library otherwise
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    res = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "host checks passed" in res.stdout
