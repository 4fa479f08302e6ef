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
    assert "ukv_trace" not in out
    # UKV_TRACE=1: one line per compute call, with the call's work-list figures; failed calls say so
    out = _run([exe, "3"], env=dict(ENV, UKV_TRACE="1"), timeout=300)
    assert "host driver ok" in out and "ERROR" not in out and "runtime error" not in out, out[-2000:]
    lines = [l for l in out.splitlines() if l.startswith("ukv_trace ")]
    calls = {l.split()[1] for l in lines}
    for call in ("call=ukv_decode_attention", "call=ukv_decode_step", "call=ukv_plan_step", "call=ukv_append",
                 "call=ukv_gather", "call=ukv_scatter", "call=ukv_prefill_attention"):
        assert call in calls, (call, sorted(calls))
    step = next(l for l in lines if "call=ukv_decode_step" in l and "status=ok" in l)
    for key in ("t_us=", "host_us=", "requests=", "kv_bytes=", "spans=", "items=", "workgroups="):
        assert key in step, step
    assert any("status=error" in l for l in lines), "the driver's rejected calls should be traced as errors"


def test_oracle_under_sanitizers(tmp_path):
    cc = shutil.which("gcc")
    if not cc:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_asan")
    _run([cc, "-std=c99", "-fopenmp", "-Wall"] + FLAGS +
         [os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "ukv_oracle.c"), "-o", exe, "-lm"])
    out = _run([exe], env=ENV, timeout=300)
    assert "oracle driver ok" in out and "ERROR" not in out and "runtime error" not in out, out[-2000:]
