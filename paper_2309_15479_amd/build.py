"""Builds liblsh.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblsh.so")
SOURCES = ["api.hip", "sampled_kernel.hip", "shared_kernel.hip", "dense_kernel.hip", "dense_split_kernel.hip", "pack_kernel.hip", "index.hip", "params_host.cpp", "schedule.cpp", "collision_law.cpp"]


def build_library(verbose=False):
    """Always recompiles; returns the path of the shared library."""
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-ffp-contract=off", "-fno-gpu-rdc",
           # keep the compiler from forming packed fp32 instructions out of scalar float code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           # device code only: no NaN bookkeeping, which lets floor + convert become one
           # instruction; vectors with NaN coordinates get unspecified ids either way
           "-Xarch_device", "-fno-honor-nans",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-Wall", "-Wno-unused-command-line-argument",
           "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True, cwd=CSRC)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
