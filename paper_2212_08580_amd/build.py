"""Compile libngc.so for gfx950 with hipcc, in-tree (next to this file).

Every source is compiled to an object of its own (in parallel) and the objects are linked;
`--host-asan` builds libngc_asan.so, the same library with its host code under
AddressSanitizer and UndefinedBehaviorSanitizer, for the CPU tests of the host logic.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libngc.so")
ASAN_LIB = os.path.join(HERE, "libngc_asan.so")
OBJ_DIR = os.path.join(HERE, "_build")
HOST_SOURCES = ["ngc_host.cpp", "ngc_solve.cpp", "ngc_latency_host.cpp"]
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


def asan_runtime():
    """Path of the sanitizer runtime the instrumented library needs preloaded into Python."""
    clang = os.path.join(os.path.dirname(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")), "..", "llvm", "bin", "clang++")
    out = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE, text=True)
    return out.stdout.strip()


def build_host_asan(verbose=True):
    """libngc_asan.so: the whole library with its HOST code under AddressSanitizer and
    UndefinedBehaviorSanitizer (device code is compiled as always; GPU sanitizers are not
    used).  For the CPU tests of the host logic: code construction, schedules, decode-vector
    selection, table sizes, latency closed forms.  Run them with
        LD_PRELOAD=<asan_runtime()> ASAN_OPTIONS=detect_leaks=0 NGC_LIB=<ASAN_LIB> \
            python -m pytest tests/test_libngc_host.py -m "not gpu"
    (the interpreter itself is not instrumented, hence the preload)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    obj_dir = os.path.join(OBJ_DIR, "asan")
    os.makedirs(obj_dir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]

    def compile_one(src):
        obj = os.path.join(obj_dir, src + ".o")
        _run([hipcc] + FLAGS + san + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj], verbose)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    _run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined",
          "-fno-gpu-sanitize", "-shared-libsan"] + objs + ["-o", ASAN_LIB], verbose)
    return ASAN_LIB


if __name__ == "__main__":
    if "--host-asan" in sys.argv[1:]:
        build_host_asan()
        print("preload for the tests:", asan_runtime())
    else:
        build_library()
    sys.exit(0)
