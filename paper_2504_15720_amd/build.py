"""Build libukv.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libukv.so")
OBJ_DIR = os.path.join(HERE, "_build")

SOURCES = ["ukv_pool.cpp", "ukv_planner.cpp", "ukv_api.cpp", "ukv_sched.cpp", "ukv_decode.hip", "ukv_prefill.hip",
           "ukv_copy.hip", "ukv_static.hip"]
# packed fp32 VALU forms are switched off for device code on this target
DEVICE_FLAGS = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# The matrix-core paths take maxima of matrix-instruction results; without this flag every operand of a maximum is
# first passed through a quieting v_max (q and the K/V of valid tokens must be finite anyway: see ukv.h).  Measured:
# prefill +2.5 %, decode within 0.5 %.
# ukv_decode.hip also keeps single-lane atomics as they are written: rewritten as a wave-wide reduction plus one
# atomic, the result is needed at once, and the take of the next span could not stay in flight behind the item.
PER_SOURCE = {"ukv_prefill.hip": ["-fno-honor-nans"],
              "ukv_decode.hip": ["-fno-honor-nans", "-mllvm", "-amdgpu-atomic-optimizer-strategy=None"]}
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument",
          "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def sources_newer_than_lib() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "ukv.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build_library(verbose: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library.  Always compiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ_DIR, src + ".o")
        cmd = [hipcc] + COMMON + DEVICE_FLAGS + PER_SOURCE.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return LIB


CALIB_DIR = os.path.join(HERE, "calib")
CALIB_PROGRAMS = [("hbm_calib", [])]
CALIB_BIN = os.path.join(CALIB_DIR, "hbm_calib")


def build_calib() -> str:
    """The stand-alone streaming copy/read program that calibrates the profiler's HBM byte counters."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    for name, extra in CALIB_PROGRAMS:
        src = name
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Wno-unused-command-line-argument"] + \
            DEVICE_FLAGS + extra + [os.path.join(CALIB_DIR, src + ".hip"), "-o", os.path.join(CALIB_DIR, name)]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {name}.hip:\n" + r.stdout)
    return CALIB_BIN


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_calib())
