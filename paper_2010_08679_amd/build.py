"""Compiles libcnr.so (the HIP kernels and their C ABI) in-tree for gfx950."""
from __future__ import annotations

import glob
import hashlib
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libcnr.so")
STAMP = LIB + ".srchash"   # hash of what LIB was built from, written next to it

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # one rounding per fp32 operation: no contraction into fused multiply-adds, no fast-math
    "-ffp-contract=off", "-fno-fast-math",
    # NaN inputs are outside the library's contract: without the IEEE mode bit the compiler need not
    # quiet signalling NaNs in front of every min / max (one extra instruction each) and can fold the
    # DPP lane exchanges of the row reductions into the min / max instructions themselves
    "-fno-honor-nans", "-mno-amdgpu-ieee",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def dependencies():
    return sources() + sorted(glob.glob(os.path.join(CSRC, "*.h"))) + [os.path.join(ROOT, "include", "cnr.h")]


def source_hash() -> str:
    """Hash of the compiler flags and of every file the library is built from."""
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    for path in dependencies():
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def is_stale() -> bool:
    """True when there is no built library, or it was built from other sources than the ones here:
    by the hash recorded at build time, or, where that record is missing, by modification times."""
    if not os.path.exists(LIB):
        return True
    if os.path.exists(STAMP):
        with open(STAMP, "r") as f:
            return f.read().strip() != source_hash()
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in dependencies())


def build_lib(force: bool = True, verbose: bool = False) -> str:
    """Runs hipcc over every .hip file under csrc/ and links them into libcnr.so."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", tmp, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    built_from = source_hash()
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    with open(STAMP, "w") as f:
        f.write(built_from + "\n")
    return LIB


if __name__ == "__main__":
    print(build_lib(force=True, verbose=True))
