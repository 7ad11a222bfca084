"""Build step: compiles csrc/*.hip for gfx950 into paper_2601_18511_amd/libpcmm.so (in-tree)."""
from __future__ import annotations

import hashlib
import os
import subprocess
import tempfile

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
# translation units of the library (each holds its own kernels; no device code crosses files)
SOURCES = [os.path.join(CSRC, n) for n in ("pcmm.hip", "pcmm_shortk.hip", "pcmm_slot.hip", "pcmv.hip")]
SRC = SOURCES[0]
HEADER = os.path.join(os.path.dirname(_HERE), "include", "pcmm.h")
INTERNAL_HEADERS = [os.path.join(CSRC, n) for n in ("pcmm_host.hpp", "pcmm_device.hpp", "pcmm_shortk.hpp", "pcmm_hip_util.hpp", "pcmv_host.hpp")]
LIB = os.path.join(_HERE, "libpcmm.so")
STAMP = LIB + ".stamp"          # digest of the sources and flags the library was built from

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
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
    for path in SOURCES + INTERNAL_HEADERS + [HEADER]:
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
    hipcc = hipcc_path()
    with tempfile.TemporaryDirectory(prefix="pcmm_build_") as tmpdir:
        objs, procs = [], []
        for src in SOURCES:      # the translation units compile side by side
            obj = os.path.join(tmpdir, os.path.basename(src) + ".o")
            objs.append(obj)
            procs.append((src, subprocess.Popen([hipcc] + HIPCC_FLAGS + ["-c", "-o", obj, src],
                                                stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        for src, proc in procs:
            out, _ = proc.communicate()
            if proc.returncode != 0:
                raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        tmp = LIB + ".tmp%d" % os.getpid()
        proc = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                              stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed to link:\n" + proc.stdout)
    os.replace(tmp, LIB)
    with open(STAMP + ".tmp%d" % os.getpid(), "w") as f:
        f.write(source_digest() + "\n")
    os.replace(STAMP + ".tmp%d" % os.getpid(), STAMP)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True))
