"""CPU builds under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU): the C flow solvers of the checker on
seeded instances, and the host side of the C ABI (api.cpp linked against stand-ins for the kernel launchers)
through its error paths and one accepted call per entry point.  Any sanitizer report aborts the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
FLAGS = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)


def run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, r.stdout[-4000:]
    return r.stdout


def test_flow_solvers_under_sanitizers(tmp_path):
    exe = str(tmp_path / "san_mcmf")
    run(["gcc", "-std=c11"] + FLAGS + [os.path.join(ROOT, "oracle", "mcmf.c"), os.path.join(SAN, "mcmf_driver.c"),
                                       "-o", exe])
    out = run([exe], env=ENV)
    assert "ok" in out


def test_host_boundary_under_sanitizers(tmp_path):
    clang = "/opt/rocm/llvm/bin/clang++"
    if not os.path.exists(clang):
        clang = shutil.which("clang++") or shutil.which("g++")
    if clang is None or not os.path.exists("/opt/rocm/include/hip/hip_runtime.h"):
        pytest.skip("no host compiler or HIP headers")
    exe = str(tmp_path / "san_host")
    run([clang, "-std=c++17", "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
         "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2508_12801_amd", "csrc")] + FLAGS +
        [os.path.join(ROOT, "paper_2508_12801_amd", "csrc", "api.cpp"), os.path.join(SAN, "host_stubs.cpp"),
         os.path.join(SAN, "host_driver.cpp"), "-o", exe])
    out = run([exe], env=ENV)
    assert "ok" in out
