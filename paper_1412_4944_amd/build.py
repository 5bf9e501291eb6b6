"""Builds libsbo.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_1412_4944_amd.build
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB_DIR = os.path.join(HERE, "lib")
LIB = os.path.join(LIB_DIR, "libsbo.so")

SOURCES = ["sbo_api.hip", "code_energy.hip", "code_select.hip", "select_accum.hip", "group.hip", "accumulate.hip",
           "polar_jacobi.hip", "polar_ns.hip", "polar_wide.hip", "polar_wide_ns.hip", "reduce.hip", "worst.hip"]
# bench.py's achievable-peak probes: a library of their own, not part of libsbo
PROBE_SOURCE = "bench_probe.hip"
PROBE_LIB = os.path.join(LIB_DIR, "libsbo_benchprobe.so")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]

# Per-source additions.  The energy kernel reads its MFMA accumulators with ordinary
# vector instructions right after each stage; keeping them in architectural VGPRs saves
# one accumulator-read instruction per value.  Its compare-exchange networks are built
# from min/max, which need no NaN-quieting pre-pass when NaNs are not honoured (signals
# or atoms holding NaN give unspecified block choices instead of propagating NaN).
EXTRA = {"code_energy.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1", "-fno-honor-nans"]}


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; libsbo needs the ROCm toolchain")
    return exe


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [hipcc(), *FLAGS, *EXTRA.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    os.makedirs(LIB_DIR, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as ex:
        objs = list(ex.map(_compile, SOURCES + [PROBE_SOURCE]))
    for out, parts in ((LIB, objs[:-1]), (PROBE_LIB, objs[-1:])):
        cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *parts, "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
        if verbose:
            print("built", out)
    return LIB


if __name__ == "__main__":
    build()
