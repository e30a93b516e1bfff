"""Compile the HIP sources of this package into libaffmae.so for gfx950.

hipcc cross-compiles without a GPU.  The library is built in-tree so that it
travels with the source tree; nothing is installed.
"""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libaffmae.so")

ARCH = "gfx950"
COMMON = ["--offload-arch=" + ARCH, "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
          # keep the compiler from forming packed-fp32 instructions
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-munsafe-fp-atomics"]
# per-file extra flags
EXTRA = {
    "knn.hip": ["-ffp-contract=off"],  # distances must not be fused
    "vts.hip": ["-ffp-contract=off"],  # likewise (grid points and table distances)
    "relpos.hip": ["-ffp-contract=off"],  # likewise (offset times bin rate)
}


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _headers_mtime() -> float:
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(HERE, "..", "include", "affmae.h"))
    return max(os.path.getmtime(h) for h in hs)


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    path = os.path.join(CSRC, src)
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= max(os.path.getmtime(path), _headers_mtime()):
        return obj
    cmd = ["hipcc", "-c", path, "-o", obj] + COMMON + EXTRA.get(src, [])
    subprocess.run(cmd, check=True)
    return obj


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile every .hip file and link libaffmae.so; returns its path."""
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), srcs))
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=" + ARCH, "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    import sys
    print(build_library(force="--incremental" not in sys.argv, verbose=True))
