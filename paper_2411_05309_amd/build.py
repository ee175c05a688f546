"""Build libgpuvm.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = [os.path.join(HERE, "csrc", f) for f in ("core.hip", "workloads.hip", "graph.hip", "phased.hip", "roofline.hip")]
LIB = os.path.join(HERE, "libgpuvm.so")

PUBLIC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-fvisibility=hidden", "-fno-gpu-rdc",
    # packed fp32 forms are not to be generated on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"),
]
FLAGS = PUBLIC_FLAGS + ["-I", os.path.join(HERE, "csrc")]


def build(verbose=False, extra=()):
    cmd = ["hipcc", *FLAGS, *extra, "-o", LIB, *SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def build_user_kernel(verbose=False):
    """The test suite's stand-in for a user's own kernel library: built from the
    public headers only and linked against libgpuvm.so."""
    src = os.path.join(ROOT, "tests", "user_kernel", "vector_add_user.hip")
    out = os.path.join(ROOT, "tests", "user_kernel", "libuser_vector_add.so")
    cmd = ["hipcc", *PUBLIC_FLAGS, "-o", out, src, "-L", HERE, "-lgpuvm",
           "-Wl,-rpath,$ORIGIN/../../paper_2411_05309_amd"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return out


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
