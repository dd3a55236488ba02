"""Compile libngc.so for gfx950 with hipcc, in-tree (next to this file)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libngc.so")
SOURCES = ["ngc_host.cpp", "ngc_solve.cpp", "ngc_device.hip", "ngc_mlp.hip", "ngc_latency.hip"]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Xarch_host", "-mavx2", "-Xarch_host", "-mfma",
         "-Wall", "-Wno-unused-function"]


def build_library(verbose=True):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-x", "hip"] + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines()
                    if "packed-fp32-ops" not in l)       # host pass does not know the feature
    if verbose and out.strip():
        print(out)
    if proc.returncode:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
