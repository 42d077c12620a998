"""Build libdare.so (HIP, gfx950) in-tree: ``python -m paper_2605_08134_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
OBJ_DIR = os.path.join(PKG_DIR, "_build")
LIB_PATH = os.path.join(PKG_DIR, "libdare.so")
BENCH_LIB_PATH = os.path.join(PKG_DIR, "libdare_bench.so")   # benchmark aids, csrc/bench/

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 instruction forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-Wall", "-Wno-unused-function",
]


def sources():
    """The product library's sources, then (under bench/) those of the benchmark aids."""
    return (sorted(f for f in os.listdir(CSRC) if f.endswith(".hip")) +
            sorted(os.path.join("bench", f) for f in os.listdir(os.path.join(CSRC, "bench")) if f.endswith(".hip")))


def _compile(src):
    obj = os.path.join(OBJ_DIR, src[:-4].replace(os.sep, "_") + ".o")
    cmd = [HIPCC] + COMMON_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    return src, obj, r


def build_library(verbose=True):
    """Compile every .hip source for gfx950 and link libdare.so and libdare_bench.so.  Always
    recompiles."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as ex:
        results = list(ex.map(_compile, sources()))
    objs, bench_objs = [], []
    for src, obj, r in results:
        noise = "packed-fp32-ops"
        err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, r.stderr))
        if verbose and err.strip():
            print(err, file=sys.stderr)
        (bench_objs if src.startswith("bench") else objs).append(obj)
    for path, group in ((LIB_PATH, objs), (BENCH_LIB_PATH, bench_objs)):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", path] + group
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library())
