"""Compile libngc.so for gfx950 with hipcc, in-tree (next to this file).

Every source is compiled to an object of its own (in parallel) and the objects are linked;
`--host-asan` builds the host-only sources with AddressSanitizer and
UndefinedBehaviorSanitizer into libngc_host_asan.so (no device code, for the CPU tests of
the host logic: code construction, schedules, decode-vector selection, latency closed forms).
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libngc.so")
ASAN_LIB = os.path.join(HERE, "libngc_host_asan.so")
OBJ_DIR = os.path.join(HERE, "_build")
HOST_SOURCES = ["ngc_host.cpp", "ngc_solve.cpp"]
DEVICE_SOURCES = ["ngc_device.hip", "ngc_codec.hip", "ngc_mlp.hip", "ngc_latency.hip"]
SOURCES = HOST_SOURCES + DEVICE_SOURCES
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Xarch_host", "-mavx2", "-Xarch_host", "-mfma",
         "-Wall", "-Wno-unused-function"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines()
                    if "packed-fp32-ops" not in l)       # host pass does not know the feature
    if verbose and out.strip():
        print(out, flush=True)
    if proc.returncode:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), proc.stdout))


def build_library(verbose=True):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    sources = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, src + ".o")
        _run([hipcc] + FLAGS + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj], verbose)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(sources))) as ex:
        objs = list(ex.map(compile_one, sources))
    _run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950"] + objs + ["-o", LIB], verbose)
    return LIB


def build_host_asan(verbose=True):
    """Host-only sources under ASan + UBSan (CPU only; the device entry points are absent)."""
    cxx = os.environ.get("CXX", "g++")
    sources = [os.path.join(CSRC, s) for s in HOST_SOURCES if os.path.exists(os.path.join(CSRC, s))]
    cmd = [cxx, "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-DNGC_HOST_ONLY",
           "-I/opt/rocm/include", "-D__HIP_PLATFORM_AMD__", "-Wall"] + sources + ["-o", ASAN_LIB]
    _run(cmd, verbose)
    return ASAN_LIB


if __name__ == "__main__":
    if "--host-asan" in sys.argv[1:]:
        build_host_asan()
    else:
        build_library()
    sys.exit(0)
