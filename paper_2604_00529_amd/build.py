"""Build libmx.so (the C-ABI library of HIP kernels) for gfx950, in-tree.

    python -m paper_2604_00529_amd.build [--force]

hipcc cross-compiles without a GPU.  The three translation units are compiled in parallel.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
BUILD = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libmx.so")
SOURCES = ["mx_api.hip", "mx_ss.hip", "mx_dense.hip", "mx_gemm.hip"]
HEADERS = ["mx_device.h", "mx_launch.h"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-I" + INCLUDE, "-I" + CSRC,
         # packed-FP32 instructions are switched off for device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _newest(paths):
    return max(os.path.getmtime(p) for p in paths)


def _compile(src):
    obj = os.path.join(BUILD, src.replace(".hip", ".o"))
    cmd = ["hipcc"] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, out))
    return obj


def build(force=False, verbose=True):
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.join(INCLUDE, "mx.h")]
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= _newest(deps):
        return LIB
    os.makedirs(BUILD, exist_ok=True)
    if verbose:
        print("[build] hipcc --offload-arch=gfx950: %s" % ", ".join(SOURCES), flush=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    if verbose:
        print("[build] wrote %s" % LIB, flush=True)
    return LIB


if __name__ == "__main__":
    build(force="--force" in sys.argv)
