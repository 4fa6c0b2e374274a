"""Compile the HIP sources in csrc/ into libmoe_mi355x.so (gfx950), in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_NAME = "libmoe_mi355x.so"
LIB_PATH = os.path.join(PKG_DIR, LIB_NAME)
PROBE_SRC = "mfma_ceiling_probe.hip"   # stand-alone measurement program, not linked into the library
PROBE_PATH = os.path.join(PKG_DIR, "mfma_ceiling_probe")
SOURCES = ["ffn_down_wide.hip", "ffn_gate_up.hip", "ffn_down.hip", "api.hip", "route.hip", "permute.hip", "pack.hip", "combine.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the library can only be built with ROCm's hipcc")
    return exe


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build_library(verbose: bool = False, extra_flags=(), jobs: int = 8) -> str:
    """Compile every translation unit (in parallel) and link them into the shared library."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(PKG_DIR, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        _run([hipcc(), *flags, *extra_flags, *inc, "-c", os.path.join(CSRC, src), "-o", obj], verbose)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH], verbose)
    return LIB_PATH


def build_probe(verbose: bool = False) -> str:
    """Compile the MFMA-rate measurement program (see its header) into an in-tree executable."""
    _run([hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          os.path.join(CSRC, PROBE_SRC), "-o", PROBE_PATH], verbose)
    return PROBE_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_probe(verbose=True))
