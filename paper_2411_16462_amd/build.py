"""Builds the HIP library (gfx950) in-tree: paper_2411_16462_amd/liblioncub.so.

hipcc cross-compiles without a GPU.  Each kernel file is compiled to an object in
parallel, then linked into one shared library that exports the C ABI declared in
include/lioncub.h.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "liblioncub.so")
SOURCES = ["lc_update_pack.hip", "lc_aggregate.hip", "lc_momentum_avg.hip", "lc_l1.hip", "lc_probe.hip", "lc_api.hip"]
HEADERS = [os.path.join(CSRC, "lc_common.hpp"), os.path.join(CSRC, "lc_launch.hpp"),
           os.path.join(ROOT, "include", "lioncub.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-fno-gpu-rdc", "-Wall", "-Wextra",
         # packed fp32 instructions stay off on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src, force, extra):
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    if force or _stale(obj, [path] + HEADERS):
        subprocess.check_call([HIPCC, *FLAGS, *extra, "-c", path, "-o", obj])
    return obj


def build(force=False, extra_flags=()):
    """Compile what is stale (everything if force) and link; returns the library path."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, list(extra_flags)), SOURCES))
    if force or _stale(LIB, objs):
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
