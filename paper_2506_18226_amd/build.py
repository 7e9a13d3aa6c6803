"""Builds the HIP library (libadsa_hip.so) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB_DIR = os.path.join(_HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libadsa_hip.so")
CEILING_PATH = os.path.join(LIB_DIR, "read_ceiling")
SOURCES = ["api.hip", "select_compact.hip", "attend.hip", "attend_gqa.hip", "vcos.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # never emit packed-fp32 VALU forms
    "-mllvm", "-amdgpu-kernarg-preload-count=16",                  # leading kernel arguments arrive in SGPRs at wave launch
    "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument",
]


def _compile_one(args):
    cmd, verbose = args
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source (one hipcc process each, side by side) and link one shared library;
    returns its path."""
    from concurrent.futures import ThreadPoolExecutor

    os.makedirs(LIB_DIR, exist_ok=True)
    obj_dir = os.path.join(LIB_DIR, "obj")
    os.makedirs(obj_dir, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    objs, jobs = [], []
    for src in SOURCES:
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        objs.append(obj)
        jobs.append(([hipcc, *flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c",
                      os.path.join(CSRC, src), "-o", obj], verbose))
    with ThreadPoolExecutor(max_workers=min(len(jobs), 6)) as pool:
        list(pool.map(_compile_one, jobs))
    _compile_one(([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH], verbose))
    # measurement aid: the plain-read ceiling the attention kernel's roofline fraction is read against
    _compile_one(([hipcc, *[f for f in flags if f != "-fPIC"], os.path.join(CSRC, "read_ceiling.hip"), "-o", CEILING_PATH],
                  verbose))
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
