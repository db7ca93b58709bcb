"""Builds libdgi.so (the C-ABI library) in-tree with hipcc for gfx950."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdgi.so")
SOURCES = ["dgi_api.hip", "dgi_graph.hip", "dgi_aggregate.hip", "dgi_gat.hip", "dgi_gemm.hip", "dgi_reorder.cpp", "dgi_reorder_gpu.hip", "dgi_partial.hip", "dgi_host.hip", "dgi_sample.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + INCLUDE, "-I" + CSRC,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _compile(src):
    obj = os.path.join(OBJ_DIR, src + ".o")
    cmd = ["hipcc", "-x", "hip", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    return obj, err


def build_library(verbose=False, extra_flags=(), lib_path=None):
    """extra_flags / lib_path: build a variant next to the product library (tuning experiments)."""
    global FLAGS, LIB
    saved = (FLAGS, LIB)
    FLAGS = [*FLAGS, *extra_flags]
    LIB = lib_path or LIB
    try:
        return _build(verbose)
    finally:
        FLAGS, LIB = saved


def _build(verbose):
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        results = list(ex.map(_compile, SOURCES))
    objs = [o for o, _ in results]
    if verbose:
        for _, err in results:
            if err.strip():
                print(err, file=sys.stderr)
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
