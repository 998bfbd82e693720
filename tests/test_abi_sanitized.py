"""The library's host code under the compiler's sanitizers: csrc/sja.hip is built once more with
-fsanitize=address,undefined on the host side only (the device code is compiled as always), and
tests/abi_sanitize_driver.cpp, built the same way, drives every argument and state check of the C
ABI through it.  Those paths return before any device work, so this runs without a GPU.  An
out-of-bounds access, a use after free, a leak or undefined behaviour in the host code ends the
run with a report; a status that differs from the documented one fails it."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/lib/llvm/bin/clang++"


@pytest.mark.skipif(shutil.which("hipcc") is None or not os.path.exists(CLANG), reason="needs the ROCm compilers")
def test_host_side_of_the_library_is_clean_under_sanitizers(tmp_path):
    lib = tmp_path / "libsja_sanitized.so"
    exe = tmp_path / "abi_sanitized"
    sanitize = ["-fsanitize=address", "-fsanitize=undefined", "-fno-omit-frame-pointer"]
    host_only = [x for flag in sanitize for x in ("-Xarch_host", flag)]
    build = subprocess.run(
        ["hipcc", "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *host_only, "-o", str(lib),
         os.path.join(ROOT, "paper_2509_19086_amd", "csrc", "sja.hip")], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-4000:]
    build = subprocess.run(
        [CLANG, "-O1", "-g", "-std=c++17", *sanitize, "-fno-sanitize-recover=all", "-Wall", "-Wextra", "-o", str(exe),
         os.path.join(ROOT, "tests", "abi_sanitize_driver.cpp"), str(lib),
         f"-Wl,-rpath,{tmp_path}", "-Wl,-rpath,/opt/rocm/lib"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert run.returncode == 0, run.stdout + run.stderr[-4000:]
    assert "host ABI checks passed" in run.stdout
