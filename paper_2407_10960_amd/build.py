"""Builds liblutq.so (HIP kernels for gfx950 + the C ABI) in-tree with hipcc.

The kernels are compiled once per (bit width, dtype) pair from the same source so that the six
translation units build in parallel.  Run as `python -m paper_2407_10960_amd.build`.
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(os.path.dirname(PKG_DIR), "include")
BUILD_DIR = os.path.join(PKG_DIR, "_build")
LIB_PATH = os.path.join(PKG_DIR, "liblutq.so")

HIP_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17",
    # packed fp32 VALU forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    f"-I{INCLUDE}", f"-I{CSRC}",
]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP toolchain is required to build liblutq.so")
    return exe


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("build step failed:\n  " + " ".join(cmd) + "\n" + out)
    return out


def build(verbose: bool = False, jobs: int | None = None) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    hipcc = _hipcc()
    steps = []
    objs = []
    for bits in (2, 3, 4):
        for dt in ("F16", "BF16"):
            obj = os.path.join(BUILD_DIR, f"kernels_b{bits}_{dt.lower()}.o")
            objs.append(obj)
            steps.append([hipcc, *HIP_FLAGS, f"-DLUTQ_INST_BITS={bits}", f"-DLUTQ_INST_DT={dt}",
                          "-c", os.path.join(CSRC, "lutq_kernels.hip"), "-o", obj])
    for src in ("lutq_api.hip", "lutq_calib.hip", "lutq_quantize.hip", "lutq_trace.hip"):
        if not os.path.exists(os.path.join(CSRC, src)):
            continue
        obj = os.path.join(BUILD_DIR, src.replace(".hip", ".o"))
        objs.append(obj)
        steps.append([hipcc, *HIP_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
    obj = os.path.join(BUILD_DIR, "lutq_pack.o")
    objs.append(obj)
    steps.append(["g++", "-O3", "-fPIC", "-std=c++17", "-fopenmp", f"-I{INCLUDE}",
                  "-c", os.path.join(CSRC, "lutq_pack.cpp"), "-o", obj])
    jobs = jobs or min(8, os.cpu_count() or 1)
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        for out in ex.map(_run, steps):
            if verbose and out.strip():
                print(out)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs, "-fopenmp"])
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
