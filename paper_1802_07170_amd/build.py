"""Builds the gfx950 shared library in-tree with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcytonmt_hip.so")
SOURCES = ["api.hip", "gemm.hip", "ce.hip", "step.hip", "misc.hip", "beam.hip"]
# -amdgpu-kernarg-preload-count: the leading kernel arguments (as many as fit into the user SGPRs, at most 14
# dwords) are delivered in registers at wavefront start instead of being fetched from the argument buffer, which
# takes about 0.6 us off the head of every kernel of the recurrences' launch chains.  Kernels keep the ordinary
# fetch as their first instructions for firmware without the feature (the compiler emits both entries).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-kernarg-preload-count=16"]


def build(verbose: bool = False) -> str:
    """Compiles every source and links the library; always recompiles.  Returns the library path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
        if verbose:
            print("compiled", src)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(one, SOURCES))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    return LIB


def ensure_built() -> str:
    """For tests, the smoke run and the benchmark: the library as it was built, or a fresh build when
    there is none.  (The binding itself never builds: without the library it raises.)"""
    return LIB if os.path.exists(LIB) else build()


if __name__ == "__main__":
    print(build(verbose=True))
