"""Build libquest.so (the C-ABI library of HIP kernels) for gfx950 with hipcc.

Usage:  python -m paper_2406_10774_amd.build
The library is built in-tree next to this file so that it travels with the
source tree; nothing is JIT-compiled at import time."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libquest.so")
BUILD_DIR = os.path.join(PKG_DIR, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


YARDSTICK_SRC = os.path.join(PKG_DIR, "bench_kernels", "yardstick.hip")
YARDSTICK_LIB = os.path.join(PKG_DIR, "libquest_yardstick.so")


def build_yardstick(verbose: bool = True) -> str:
    """The benchmark's own kernels (plain reads, a bare gather): a library of its own."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    tmp = YARDSTICK_LIB + ".tmp"
    r = subprocess.run([hipcc, *HIPCC_FLAGS, "-shared", YARDSTICK_SRC, "-o", tmp],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {YARDSTICK_SRC}:\n{r.stderr}")
    os.replace(tmp, YARDSTICK_LIB)
    if verbose:
        print(f"built {YARDSTICK_LIB}")
    return YARDSTICK_LIB


def build(verbose: bool = True) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    os.makedirs(BUILD_DIR, exist_ok=True)
    build_yardstick(verbose)

    def compile_one(src):
        obj = os.path.join(BUILD_DIR, os.path.basename(src)[:-4] + ".o")
        cmd = [hipcc, *HIPCC_FLAGS, "-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        noise = "is not a recognized feature for this target"
        err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as ex:
        objs = list(ex.map(compile_one, sources()))
    tmp = LIB_PATH + ".tmp"
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    os.replace(tmp, LIB_PATH)
    if verbose:
        print(f"built {LIB_PATH}")
    return LIB_PATH


if __name__ == "__main__":
    build()
