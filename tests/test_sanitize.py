"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

Two programs are built here and run: the library's host side (pool, planner, scheduler, argument checks, staging of
every compute call) against stand-ins for the HIP calls and kernel launches that walk what the kernels would read
(tests/sanitize/fake_hip_and_launchers.cpp, ukv_host_driver.cpp); and the CPU oracle with its own driver
(oracle_driver.c).  A sanitizer report makes the program exit with an error.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
CSRC = os.path.join(ROOT, "paper_2504_15720_amd", "csrc")
FLAGS = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd[:3])} ... failed:\n{r.stdout[-4000:]}"
    return r.stdout


def test_library_host_code_under_sanitizers(tmp_path):
    cxx = "/opt/rocm/llvm/bin/clang++" if os.path.exists("/opt/rocm/llvm/bin/clang++") else shutil.which("clang++")
    if not cxx:
        pytest.skip("no clang++")
    exe = str(tmp_path / "ukv_host_asan")
    srcs = [os.path.join(SAN, "ukv_host_driver.cpp"), os.path.join(SAN, "fake_hip_and_launchers.cpp")] + \
        [os.path.join(CSRC, f) for f in ("ukv_pool.cpp", "ukv_planner.cpp", "ukv_api.cpp", "ukv_sched.cpp")]
    _run([cxx, "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"),
          "-I" + CSRC, "-Wno-unused-result", "-Wno-unknown-attributes"] + FLAGS + srcs + ["-o", exe])
    out = _run([exe, "40"], env=ENV, timeout=300)
    assert "host driver ok" in out and "ERROR" not in out and "runtime error" not in out, out[-2000:]


def test_oracle_under_sanitizers(tmp_path):
    cc = shutil.which("gcc")
    if not cc:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_asan")
    _run([cc, "-std=c99", "-fopenmp", "-Wall"] + FLAGS +
         [os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "ukv_oracle.c"), "-o", exe, "-lm"])
    out = _run([exe], env=ENV, timeout=300)
    assert "oracle driver ok" in out and "ERROR" not in out and "runtime error" not in out, out[-2000:]
