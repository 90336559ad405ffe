"""Builds libstencil.so (hipcc, gfx950) in-tree, next to this file."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "_lib", "libstencil.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-ffp-contract=off",                       # fma only where the source says fma
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]
OBJ_DIR = os.path.join(_HERE, "_lib", "_build")


def sources():
    return [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".hip")]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # hipcc's host pass does not know the packed-fp32 feature and says so: harmless
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False, extra_flags=(), jobs: int = 0) -> str:
    """Compiles every translation unit of csrc/ (in parallel) and links libstencil.so."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    tag = ".%d" % os.getpid()
    srcs = sources()
    objs = [os.path.join(OBJ_DIR, os.path.basename(s)[:-4] + tag + ".o") for s in srcs]
    tmp = LIB_PATH + ".tmp" + tag
    jobs = jobs or min(len(srcs), max(1, (os.cpu_count() or 2) - 1), 8)
    try:
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            list(pool.map(lambda so: _run([hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-c", so[0], "-o", so[1]], verbose),
                          zip(srcs, objs)))
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp], verbose)
        os.replace(tmp, LIB_PATH)
    finally:
        for f in objs + [tmp]:
            if os.path.exists(f):
                os.remove(f)
    return LIB_PATH


EXAMPLE_SRC = os.path.join(os.path.dirname(_HERE), "examples", "heat_sweep.cpp")
EXAMPLE_BIN = os.path.join(os.path.dirname(_HERE), "examples", "_build", "heat_sweep")


def build_example(verbose: bool = False) -> str:
    """Compiles examples/heat_sweep.cpp (plain C++ against include/libstencil.h) and links it with
    the library just built; the binary finds the library relative to itself."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(os.path.dirname(EXAMPLE_BIN), exist_ok=True)
    _run([hipcc, "-O2", "-std=c++17", EXAMPLE_SRC, "-I" + os.path.join(os.path.dirname(_HERE), "include"),
          "-L" + os.path.dirname(LIB_PATH), "-lstencil", "-Wl,-rpath,$ORIGIN/../../paper_1511_02490_amd/_lib",
          "-o", EXAMPLE_BIN], verbose)
    return EXAMPLE_BIN


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
