"""Builds liblsh.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "liblsh.so")
SOURCES = ["api.hip", "sampled_kernel.hip", "ranged_kernel.hip", "shared_kernel.hip", "shared_ranged_kernel.hip", "dense_kernel.hip",
           "dense_split_kernel.hip", "dense_split_wide_kernel.hip", "pack_kernel.hip", "index.hip", "params_host.cpp", "schedule.cpp",
           "collision_law.cpp", "selfcheck.cpp"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-ffp-contract=off", "-fno-gpu-rdc",
         # keep the compiler from forming packed fp32 instructions out of scalar float code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # device code only: no NaN bookkeeping, which lets floor + convert become one
         # instruction; vectors with NaN coordinates get unspecified ids either way
         "-Xarch_device", "-fno-honor-nans",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC,
         "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]


def _newest_header():
    heads = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    heads.append(os.path.join(ROOT, "include", "lsh.h"))
    return max(os.path.getmtime(h) for h in heads)


def build_library(verbose=False, incremental=False, jobs=None):
    """Compiles every source (all of them unless incremental, then only those older than their
    object file) and links the shared library; returns its path."""
    os.makedirs(OBJ, exist_ok=True)
    heads = _newest_header()
    todo = []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s + ".o")
        fresh = (incremental and os.path.exists(obj)
                 and os.path.getmtime(obj) > max(os.path.getmtime(src), heads, os.path.getmtime(__file__)))
        if not fresh:
            # .cpp files hold host code only, but go through hipcc as HIP sources too so that one
            # set of flags serves all
            todo.append(["hipcc", "-x", "hip", "-c", src, "-o", obj] + FLAGS)

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, cwd=CSRC, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        return cmd, r

    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        for cmd, r in pool.map(run, todo):
            out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
            if r.returncode != 0:
                sys.stderr.write(out + "\n")
                raise subprocess.CalledProcessError(r.returncode, cmd)
            if verbose and out.strip():
                print(out)
    link = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", LIB] + \
           [os.path.join(OBJ, s + ".o") for s in SOURCES]
    subprocess.run(link, check=True, cwd=CSRC)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv, incremental="-i" in sys.argv))
