"""Host side of libdisco under AddressSanitizer + UndefinedBehaviorSanitizer (CPU tier; never run on a GPU
box: sanitizers instrument HOST code only, `-Xarch_host -fsanitize=...`).  Builds an instrumented copy of the
library next to a small C++ driver that walks the boundary's host paths (handle creation and destruction,
page-order validation, every call's argument checks, the host-only arithmetic), runs the driver and fails on
any unexpected result or sanitizer report."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2405_04304_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANGXX = "/opt/rocm/llvm/bin/clang++"


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANGXX)), reason="ROCm toolchain not installed")
def test_host_paths_clean_under_asan_and_ubsan(tmp_path):
    lib = tmp_path / "libdisco_san.so"
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all",
           "-Xarch_host", "-fno-omit-frame-pointer"]
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-x", "hip",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", os.path.join(ROOT, "include")] + san + [
           os.path.join(CSRC, "disco_kernels.hip"), os.path.join(CSRC, "disco_api.cpp"), "-o", str(lib)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    exe = tmp_path / "driver"
    r = subprocess.run([CLANGXX, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                        "-fno-omit-frame-pointer", os.path.join(ROOT, "tests", "host_sanitizers", "driver.cpp"), str(lib),
                        "-Wl,-rpath," + str(tmp_path), "-Wl,-rpath,/opt/rocm/lib", "-o", str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ)
    # the HIP runtime keeps process-lifetime allocations of its own: leak reports are limited to this library's frames
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert r.returncode == 0 and "ok: 0 unexpected results" in out, out[-4000:]
