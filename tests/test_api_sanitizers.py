"""The library's host code (argument checks, segment handling, options) under AddressSanitizer and
UndefinedBehaviorSanitizer.  Only the host pass is instrumented (device code cannot be on this
hardware pool); the driver makes calls that are answered on the host, so no GPU is needed."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANGXX = "/opt/rocm/llvm/bin/clang++"


def test_host_side_of_the_library_is_clean_under_asan_and_ubsan(tmp_path):
    if not (os.path.exists(HIPCC) and os.path.exists(CLANGXX)):
        pytest.skip("ROCm compilers not available")
    csrc = os.path.join(ROOT, "paper_2405_17517_amd", "csrc")
    lib = str(tmp_path / "libwash_asan.so")
    build = subprocess.run(
        [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined"]
        + [os.path.join(csrc, f) for f in ("api.hip", "shuffle.hip", "reduce.hip", "diagnostics.hip")] + ["-o", lib],
        capture_output=True, text=True, timeout=900)
    assert build.returncode == 0, build.stderr[-3000:]
    exe = str(tmp_path / "api_sanitize")
    link = subprocess.run(
        [CLANGXX, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         os.path.join(ROOT, "tests", "api_sanitize_driver.cpp"), "-o", exe, "-L" + str(tmp_path), "-lwash_asan",
         "-Wl,-rpath," + str(tmp_path)], capture_output=True, text=True, timeout=300)
    assert link.returncode == 0, link.stderr[-3000:]
    env = dict(os.environ)
    # the HIP runtime keeps allocations for the life of the process: leak checking would only report those
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert "all checks passed" in run.stdout
