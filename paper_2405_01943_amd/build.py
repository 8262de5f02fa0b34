"""Build libdass.so (HIP, gfx950) in-tree.  Run as ``python -m paper_2405_01943_amd.build``.

Every source is compiled to an object of its own (in parallel) and the objects are linked into
``libdass.so``.  Beside the library a small text file records the SHA-256 of the sources it was
built from; ``is_stale()`` compares that with the sources as they are now, so a library older than
its sources is noticed whatever the file times say.
"""
from __future__ import annotations

import glob
import hashlib
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
INCLUDE = os.path.join(_HERE, "..", "include")
LIB = os.path.join(_HERE, "libdass.so")
STAMP = LIB + ".sources"          # SHA-256 of the sources LIB was built from
OBJ_DIR = os.path.join(_HERE, "_build")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # packed-f32 VALU forms are kept out of generated code on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-munsafe-fp-atomics",  # f32 atomic add in hardware instead of a CAS loop
    "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _dependencies():
    return sources() + sorted(glob.glob(os.path.join(CSRC, "*.h"))) + sorted(glob.glob(os.path.join(INCLUDE, "*.h")))


def source_hash() -> str:
    """SHA-256 over names and contents of every file the library is built from, and the flags."""
    h = hashlib.sha256()
    h.update(" ".join(HIPCC_FLAGS).encode())
    for path in _dependencies():
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def is_stale() -> bool:
    """True when libdass.so is missing or was built from other sources than the present ones."""
    if not os.path.exists(LIB) or not os.path.exists(STAMP):
        return True
    with open(STAMP) as f:
        return f.read().strip() != source_hash()


def build(verbose: bool = False, jobs: int = 8) -> str:
    """Compile every HIP source and link libdass.so; raises on failure."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    digest = source_hash()
    if os.path.exists(STAMP):
        os.remove(STAMP)          # no stamp while the library is being replaced

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        cmd = [hipcc] + HIPCC_FLAGS + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        objects = list(pool.map(compile_one, sources()))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objects
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    with open(STAMP, "w") as f:
        f.write(digest + "\n")
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    print("built", LIB)
    sys.exit(0)
