"""The host side of the library under AddressSanitizer + UndefinedBehaviorSanitizer, on the CPU.

Builds the library once more with the sanitizers on its host code (device code is compiled as usual and never
runs here), links a small C++ driver that walks the C ABI's workspace queries and argument checks, and runs it: any
out-of-bounds access, use after free or undefined arithmetic in the argument validation, the workspace planning or
the error plumbing aborts the driver.  GPU sanitizers are not available on the test machines; this covers the host.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2509_10771_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANGXX = os.environ.get("CLANGXX", "/opt/rocm/lib/llvm/bin/clang++")
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
       "-Xarch_host", "-fno-omit-frame-pointer"]
SOURCES = ["gemm.hip", "fused_forward.hip", "elementwise.hip", "recurrent.hip", "api.hip", "api_recurrent.hip"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), r.stdout[-4000:], r.stderr[-4000:])
    return r


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_host_side_under_address_and_ub_sanitizers(tmp_path):
    def compile_one(src):
        obj = str(tmp_path / src.replace(".hip", ".o"))
        _run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
              "-packed-fp32-ops"] + SAN + ["-c", os.path.join(CSRC, src), "-o", obj])
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    lib = str(tmp_path / "librslx_san.so")
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined", "-shared-libsan",
          "-o", lib] + objs)
    exe = str(tmp_path / "host_driver")
    _run([CLANGXX, "-std=c++17", "-g", "-O1", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined",
          "-shared-libsan", os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp"), "-o", exe, lib, "-Wl,-rpath," + str(tmp_path)])
    env = dict(os.environ)
    rt = subprocess.run([CLANGXX, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    env["LD_LIBRARY_PATH"] = os.path.dirname(rt) + os.pathsep + env.get("LD_LIBRARY_PATH", "")
    # the HIP runtime keeps process-lifetime allocations: leak checking off; everything else at its default
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    sys.stdout.write(r.stdout[-3000:])
    assert r.returncode == 0, "%s\n%s" % (r.stdout[-4000:], r.stderr[-6000:])
    assert "all checks passed" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-6000:]
