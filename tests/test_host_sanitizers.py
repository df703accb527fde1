"""The library's host code (argument checks, workspace carve-up, launch-shape choice) under the address
and undefined-behaviour sanitizers, on the CPU: a sanitizer build of every source (host side
instrumented, device side compiled without optimisation since it never runs here) is linked into a
library of its own under the test's temporary folder, and tests/c/abi_checks.c, built with the same
sanitizers, drives every entry point through its rejections."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# host code only: the device side is never instrumented (and never runs here)
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
SAN_HOST_ONLY = ["-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-shared-libsan"]


def test_argument_checks_under_address_and_undefined_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clang = "/opt/rocm/llvm/bin/clang"
    if not (os.path.exists(hipcc) and os.path.exists(clang)):
        pytest.skip("no ROCm compiler here")
    from paper_2405_12591_amd import build as B
    inc = ["-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2405_12591_amd", "csrc")]

    def compile_one(src):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-Xarch_device", "-O0", "-std=c++17", "-fPIC", "-g",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *SAN, *inc, "-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        return obj

    with ThreadPoolExecutor(min(8, os.cpu_count() or 1)) as pool:
        objs = list(pool.map(compile_one, B.sources()))
    lib = str(tmp_path / "libdecoquant_san.so")
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *SAN_HOST_ONLY, *objs, "-o", lib],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    exe = str(tmp_path / "abi_checks")
    r = subprocess.run([clang, "-std=c99", "-g", *SAN_HOST_ONLY, "-Wno-unused-command-line-argument",
                        os.path.join(ROOT, "tests", "c", "abi_checks.c"), "-I", os.path.join(ROOT, "include"),
                        lib, "-Wl,-rpath," + str(tmp_path), "-Wl,-rpath,/opt/rocm/lib", "-o", exe],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    rt = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               LD_LIBRARY_PATH=os.path.dirname(rt) + ":/opt/rocm/lib:" + os.environ.get("LD_LIBRARY_PATH", ""))
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0 and "abi checks ok" in run.stdout, (run.stdout + run.stderr)[-4000:]
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-4000:]
