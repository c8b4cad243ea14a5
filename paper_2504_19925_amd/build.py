"""Builds libsymi.so (gfx950) in-tree with hipcc.  `python -m paper_2504_19925_amd.build`."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsymi.so")
# microbenchmarks of the part's ceilings (bench.py --ceiling): a library of their own, so that
# nothing of them is part of the product's ABI
CEILINGS_LIB = os.path.join(HERE, "libsymi_ceilings.so")
SOURCES = ["api.hip", "route.hip", "place.hip", "dispatch.hip", "gemm.hip", "adam.hip", "comm_plan.hip", "router.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    cmd = [hipcc] + FLAGS + [os.path.join(CSRC, "ceilings.hip"), "-o", CEILINGS_LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
