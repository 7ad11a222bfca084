"""Build step: compiles csrc/pcmm.hip for gfx950 into paper_2601_18511_amd/libpcmm.so (in-tree)."""
from __future__ import annotations

import hashlib
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "csrc", "pcmm.hip")
HOST_HEADER = os.path.join(_HERE, "csrc", "pcmm_host.hpp")
DEVICE_HEADER = os.path.join(_HERE, "csrc", "pcmm_device.hpp")
HEADER = os.path.join(os.path.dirname(_HERE), "include", "pcmm.h")
LIB = os.path.join(_HERE, "libpcmm.so")
STAMP = LIB + ".stamp"          # digest of the sources and flags the library was built from

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


def source_digest() -> str:
    """Digest of everything the library is built from: the sources, the headers and the flags."""
    h = hashlib.sha256()
    for path in (SRC, HOST_HEADER, DEVICE_HEADER, HEADER):
        with open(path, "rb") as f:
            h.update(f.read())
    h.update(" ".join(HIPCC_FLAGS).encode())
    return h.hexdigest()


def is_current() -> bool:
    """True if libpcmm.so exists and was built from the sources as they are now."""
    if not (os.path.exists(LIB) and os.path.exists(STAMP)):
        return False
    with open(STAMP) as f:
        return f.read().strip() == source_digest()


def build_library(force: bool = True) -> str:
    """Compile the HIP library. With force=False a libpcmm.so built from the present sources is kept."""
    if not force and is_current():
        return LIB
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc_path()] + HIPCC_FLAGS + ["-o", tmp, SRC]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    os.replace(tmp, LIB)
    with open(STAMP + ".tmp%d" % os.getpid(), "w") as f:
        f.write(source_digest() + "\n")
    os.replace(STAMP + ".tmp%d" % os.getpid(), STAMP)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True))
