"""Builds libspmoe.so (HIP kernels + host runtime, gfx950 only) in-tree with hipcc."""
import os
import subprocess

_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_DIR)
LIB = os.path.join(_DIR, "libspmoe.so")
SOURCES = [os.path.join(_DIR, "csrc", "spmoe_kernels.hip"), os.path.join(_DIR, "csrc", "spmoe_static.hip"),
           os.path.join(_DIR, "csrc", "spmoe_runtime.cpp")]


def build(verbose=False):
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fopenmp",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument",
           "-x", "hip",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(_DIR, "csrc")] + SOURCES + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
