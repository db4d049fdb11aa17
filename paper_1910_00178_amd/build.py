"""Compile the HIP library (hipcc, gfx950) in-tree.  `python -m paper_1910_00178_amd.build`."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "ngemm.hip")
LIB = os.path.join(HERE, "libngemm.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off", "-fPIC", "-shared", "-std=c++17",
    "-I" + os.path.join(ROOT, "include"),
    "-Wall", "-Wextra", "-Wno-pass-failed",
    "-Wl,--no-undefined",        # a kernel the host pass failed to emit must fail the build, not the first load
]


def _compile(src, lib, verbose):
    cmd = [HIPCC, *FLAGS, "-o", lib, src]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return lib


def build_library(verbose=False):
    return _compile(SRC, LIB, verbose)


if __name__ == "__main__":
    print(build_library(verbose=True))
    sys.exit(0)
