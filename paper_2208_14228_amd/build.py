"""Builds libes.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import hashlib
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libes.so")
STAMP = LIB + ".srchash"
SOURCES = [os.path.join(CSRC, "es_kernels.hip"), os.path.join(CSRC, "es_api.cpp"),
           os.path.join(CSRC, "es_sched.cpp")]
HEADERS = [os.path.join(CSRC, "es_internal.h"), os.path.join(ROOT, "include", "es.h"),
           os.path.join(ROOT, "include", "es_sched.h")]

# -ffp-contract=off: no fused multiply-add may be formed (bit-exact SGD update)
# -fhip-fp32-correctly-rounded-divide-sqrt: IEEE division for the /N
# -fno-gpu-flush-denormals-to-zero: fp32 denormals are kept
# packed-fp32 instructions are switched off for the device code
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-fno-gpu-flush-denormals-to-zero", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    return "hipcc"


def source_hash() -> str:
    """Identifies what a library was built from: the sources, the headers and the flags."""
    h = hashlib.sha256(" ".join(f for f in FLAGS if not os.path.isabs(f)).encode())
    for f in SOURCES + HEADERS:
        with open(f, "rb") as fh:
            h.update(os.path.basename(f).encode() + b"\0" + fh.read())
    return h.hexdigest()[:16]


def stale() -> bool:
    """True if there is no built library, or it was built from other sources than the tree holds
    (the hash of what it was built from sits beside it and is compiled into es_version())."""
    try:
        with open(STAMP) as fh:
            return not os.path.exists(LIB) or fh.read().strip() != source_hash()
    except OSError:
        return True


def build(force: bool = True, verbose: bool = False) -> str:
    if force or stale():
        tag = source_hash()
        cmd = [hipcc(), *FLAGS, f'-DES_SOURCE_HASH="{tag}"', *SOURCES, "-o", LIB]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        with open(STAMP, "w") as fh:
            fh.write(tag + "\n")
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
