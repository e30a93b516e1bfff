"""Compile the HIP sources of this package into libaffmae.so for gfx950.

hipcc cross-compiles without a GPU.  The library is built in-tree so that it
travels with the source tree; nothing is installed.
"""
from __future__ import annotations

import hashlib
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libaffmae.so")
# the same sources with per-kernel event timing compiled in (include/affmae_timing.h): loaded by the benchmark only
LIB_TIMED = os.path.join(HERE, "libaffmae_timed.so")

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


def source_id() -> str:
    """Hex digest over the library's sources (csrc/*.hip, csrc/*.h, include/*.h): compiled into the library
    (affmae_build_id) so that stored profiles can be matched to the build they were taken from."""
    h = hashlib.sha256()
    files = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".hip", ".h"))]
    inc = os.path.join(HERE, "..", "include")
    files += [os.path.join(inc, f) for f in sorted(os.listdir(inc)) if f.endswith(".h")]
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def _headers_mtime() -> float:
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(HERE, "..", "include", "affmae.h"))
    hs.append(os.path.join(HERE, "..", "include", "affmae_timing.h"))
    return max(os.path.getmtime(h) for h in hs)


def _compile(src: str, force: bool, timed: bool = False) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".timed.o" if timed else ".o"))
    path = os.path.join(CSRC, src)
    stamped = src == "api.hip"  # carries the digest of all sources: rebuilt whenever it is asked for
    if (not force and not stamped and os.path.exists(obj)
            and os.path.getmtime(obj) >= max(os.path.getmtime(path), _headers_mtime())):
        return obj
    cmd = ["hipcc", "-c", path, "-o", obj] + COMMON + EXTRA.get(src, []) + (["-DAFFMAE_TIMING"] if timed else [])
    if stamped:
        cmd.append('-DAFFMAE_BUILD_ID="%s"' % source_id())
    subprocess.run(cmd, check=True)
    return obj


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile every .hip file and link libaffmae.so and its instrumented twin libaffmae_timed.so; returns the
    path of the product library."""
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    jobs = [(s, False) for s in srcs] + [(s, True) for s in srcs]
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(lambda j: _compile(j[0], force, j[1]), jobs))
    for lib, group in ((LIB, objs[:len(srcs)]), (LIB_TIMED, objs[len(srcs):])):
        cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=" + ARCH, "-o", lib] + group
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    import sys
    print(build_library(force="--incremental" not in sys.argv, verbose=True))
