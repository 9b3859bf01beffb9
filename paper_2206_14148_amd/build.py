"""Builds libknn_mi355x.so (gfx950) in-tree with hipcc.  No JIT, no torch extension."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
OBJ_DIR = os.path.join(PKG_DIR, "_build")
LIB_PATH = os.path.join(PKG_DIR, "libknn_mi355x.so")
SOURCES = ["planner.cpp", "api.hip", "knn_lowd.hip", "knn_norms.hip", "knn_split.hip", "knn_packed.hip", "knn_wide.hip", "knn_refine.hip", "knn_peak.hip",
           "kmv_api.hip", "kmv_kernels.hip", "sgpr_api.hip", "sgpr_kernels.hip"]
HEADERS = ["knn_config.h", "knn_device.h", "knn_exact.h", "knn_kernels.h", "kmv_kernels.h", "sgpr_kernels.h",
           os.path.join("..", "..", "include", "sgpr.h"),
           os.path.join("..", "..", "include", "knn.h"),
           os.path.join("..", "..", "include", "kmv.h")]

FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         # packed fp32 VALU forms are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA results go to ordinary VGPRs so the filter reads them without copies
         "-mllvm", "-amdgpu-mfma-vgpr-form=1",
         # the chunk loop of the register-resident-query kernel must unroll completely
         "-mllvm", "-pragma-unroll-threshold=100000",
         "-Wno-unused-command-line-argument"]


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > built for f in SOURCES + HEADERS)


def build(verbose: bool = False) -> str:
    """Always compiles every source (one hipcc process each), links, returns the library path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)

    def compile_one(name: str) -> str:
        obj = os.path.join(OBJ_DIR, os.path.splitext(name)[0] + ".o")
        cmd = [hipcc] + FLAGS + ["-c", os.path.join(CSRC, name), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
