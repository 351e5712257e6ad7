"""Builds librls.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librls.so")
SOURCES = ["rls_api.hip", "gbt_score.hip", "kmeans_seed.hip", "kmeans_lloyd.hip", "snap.hip", "modes_visited.hip",
           "sweep_static.hip"]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, "rls_internal.h"), os.path.join(ROOT, "include", "rls.h"),
                        os.path.join(ROOT, "include", "rls_bench.h")]
    return any(os.path.getmtime(p) > t for p in deps)


def build_library(verbose: bool = False) -> str:
    """Compile every kernel file for gfx950 and link the shared library. Always compiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
           "-ffp-contract=off", "-mllvm", "-amdgpu-mfma-vgpr-form",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", LIB] + sources()
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(line for line in res.stderr.splitlines() if noise not in line)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
