"""The CPU oracle and the trace tools under AddressSanitizer and UndefinedBehaviorSanitizer: a small C
driver (oracle/sanitize_driver.c) calls every entry point on seeded inputs with the edge cases; built
as a stand-alone executable with gcc -fsanitize=address,undefined -fno-sanitize-recover, so any
out-of-bounds access, signed overflow or misaligned access ends it with a report."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_and_trace_tools_are_clean_under_asan_and_ubsan(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "sanitize_driver")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", exe,
           os.path.join(ROOT, "oracle", "sanitize_driver.c"), os.path.join(ROOT, "oracle", "dlrm_oracle.c"),
           os.path.join(ROOT, "workloads", "trace_tools.c"), "-lm"]
    b = subprocess.run(cmd, capture_output=True, text=True)
    if b.returncode != 0 and "asan" in (b.stderr or "").lower() and "cannot find" in b.stderr.lower():
        pytest.skip("sanitizer runtime not installed")
    assert b.returncode == 0, b.stderr[-3000:]
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "sanitize_driver ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_host_side_of_the_library_is_clean_under_asan_and_ubsan(tmp_path):
    """The method's library built once more with both sanitizers on its host code (argument checks, workspace
    layout, launch geometry) and driven through the C ABI by tests/abi_host_driver.c: every call must be
    rejected on the host with its documented status, with no sanitizer report.  Needs no GPU."""
    from paper_1906_00091_amd import build as hip_build
    clang = "/opt/rocm/lib/llvm/bin/clang"
    if not os.path.exists(clang):
        pytest.skip("no ROCm clang")
    lib = hip_build.build_host_sanitized(str(tmp_path / "hostsan"))
    exe = str(tmp_path / "abi_host_driver")
    cmd = [clang, "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-I", os.path.join(ROOT, "include"), "-o", exe, os.path.join(ROOT, "tests", "abi_host_driver.c"),
           lib, "-Wl,-rpath," + os.path.dirname(lib)]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stderr[-3000:]
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0:protect_shadow_gap=0"   # (the HIP runtime reserves address space of its own)
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "abi_host_driver ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
