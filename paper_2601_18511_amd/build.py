"""Build step: compiles csrc/pcmm.hip for gfx950 into paper_2601_18511_amd/libpcmm.so (in-tree)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "csrc", "pcmm.hip")
HEADER = os.path.join(os.path.dirname(_HERE), "include", "pcmm.h")
LIB = os.path.join(_HERE, "libpcmm.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    "-Wall",
    # the epilogue relies on exactly the double-precision operations it spells out
    "-ffp-contract=off",
    # hipcc -O3 may otherwise fuse float code into packed-fp32 forms; keep them off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build_library(force: bool = True) -> str:
    """Compile the HIP library. With force=False an up-to-date libpcmm.so is kept."""
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(SRC), os.path.getmtime(HEADER))
        if os.path.getmtime(LIB) >= newest:
            return LIB
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc_path()] + HIPCC_FLAGS + ["-o", tmp, SRC]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True))
