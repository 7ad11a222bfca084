"""ctypes loader for oracle/pcmv_oracle.c (test infrastructure; never imported by the product path).

The arithmetic lives in the C file; this module only compiles it with gcc, marshals numpy arrays and
checks shapes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pcmv_oracle.c")
_LIB = os.path.join(_HERE, "libpcmv_oracle.so")
_lib = None


def build_pcmv_oracle(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C + OpenMP). Returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", tmp, _SRC]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # PCMV_ORACLE_LIB names another build of the same pcmv_oracle.c (a sanitizer build, for instance)
        lib = ctypes.CDLL(os.environ.get("PCMV_ORACLE_LIB") or build_pcmv_oracle())
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.pcmv_oracle_select.argtypes = [p, p, p, i64, i64, i64, i64, p, i64, p]
        lib.pcmv_oracle_select.restype = ctypes.c_int
        _lib = lib
    return _lib


def pcmv_oracle_rows(pt, ct, primes, rows: Sequence[int]) -> np.ndarray:
    """out[j][r][c] = sum_k pt[rows[r]][k] * ct[j][k][c] in Z_{q_j}[X]/(X^N+1); returns uint64 [L][len(rows)][2][N].

    pt: signed integers [Mp][Kp][N];  ct: uint64 residues [L][Kp][2][N], limb j reduced mod primes[j]."""
    pt = np.ascontiguousarray(np.asarray(pt), dtype=np.int64)
    ct = np.ascontiguousarray(np.asarray(ct), dtype=np.uint64)
    q = np.ascontiguousarray(np.asarray([int(x) for x in primes], dtype=np.uint64))
    if pt.ndim != 3 or ct.ndim != 4 or ct.shape[2] != 2:
        raise ValueError("pt must be [Mp][Kp][N] and ct must be [L][Kp][2][N]")
    Mp, Kp, N = pt.shape
    L = ct.shape[0]
    if ct.shape[1] != Kp or ct.shape[3] != N or q.shape[0] != L:
        raise ValueError("shape mismatch between pt, ct and the prime list")
    if np.abs(pt).max(initial=0) >= (1 << 31):
        raise ValueError("plaintext coefficients must be below 2^31 in magnitude")
    for j in range(L):
        if ct[j].size and int(ct[j].max()) >= int(q[j]):
            raise ValueError("ct[%d] holds a residue that is not reduced mod q_j" % j)
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    out = np.empty((L, rows.size, 2, N), dtype=np.uint64)
    rc = _load().pcmv_oracle_select(pt.ctypes.data, ct.ctypes.data, q.ctypes.data, Mp, Kp, N, L,
                                    rows.ctypes.data, rows.size, out.ctypes.data)
    if rc != 0:
        raise RuntimeError("pcmv_oracle_select failed (index out of range?)")
    return out


def pcmv_oracle(pt, ct, primes) -> np.ndarray:
    """All output polynomials: uint64 [L][Mp][2][N]."""
    return pcmv_oracle_rows(pt, ct, primes, np.arange(np.asarray(pt).shape[0]))
