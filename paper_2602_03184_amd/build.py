"""Builds libdsk.so (the HIP kernels + C ABI) in-tree for gfx950 with hipcc.

    python paper_2602_03184_amd/build.py

Objects go to paper_2602_03184_amd/_build/, the library to paper_2602_03184_amd/libdsk.so.
Beside it: the host-only C example (dsk_example) and libdsk_benchaid.so, a streaming-read
yardstick that only bench.py loads (it is not part of the library).
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
BUILD_DIR = os.path.join(PKG_DIR, "_build")
LIB_PATH = os.path.join(PKG_DIR, "libdsk.so")
EXAMPLE_SRC = os.path.join(PKG_DIR, "examples", "dsk_example.cpp")
EXAMPLE_PATH = os.path.join(PKG_DIR, "dsk_example")
BENCHAID_SRC = os.path.join(PKG_DIR, "benchaid", "stream_read_probe.hip")
BENCHAID_PATH = os.path.join(PKG_DIR, "libdsk_benchaid.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-fvisibility=hidden",
    "-Wall",
    "-Wno-unused-function",
    # packed fp32 VALU forms are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the DynSplit-KV HIP library cannot be built")
    return exe


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str) -> str:
    obj = os.path.join(BUILD_DIR, os.path.basename(src)[:-4] + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if "warning" in warn:
        sys.stderr.write(warn + "\n")
    return obj


def build_library(jobs: int = 8) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, sources()))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    build_example()
    build_benchaid()
    return LIB_PATH


def build_benchaid() -> str:
    """The benchmark's streaming-read yardstick: one source file, its own shared object."""
    cmd = [_hipcc(), *HIPCC_FLAGS, "-shared", BENCHAID_SRC, "-o", BENCHAID_PATH]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("building the bench aid failed:\n%s\n%s" % (r.stdout, r.stderr))
    return BENCHAID_PATH


def build_example() -> str:
    """The host-only example on the C ABI (no Python, no torch), linked against the library beside it."""
    cmd = [_hipcc(), "--offload-arch=gfx950", "-O2", "-std=c++17", "-I", os.path.join(os.path.dirname(PKG_DIR), "include"),
           EXAMPLE_SRC, "-L", PKG_DIR, "-ldsk", "-Wl,-rpath,$ORIGIN", "-o", EXAMPLE_PATH]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("building the example failed:\n%s\n%s" % (r.stdout, r.stderr))
    return EXAMPLE_PATH


if __name__ == "__main__":
    print(build_library())
