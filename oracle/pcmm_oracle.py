"""ctypes loader for oracle/pcmm_oracle.c (test infrastructure; never imported by the product path).

The arithmetic lives in the C file; this module only compiles it with gcc,
marshals numpy arrays and checks shapes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pcmm_oracle.c")
_LIB = os.path.join(_HERE, "libpcmm_oracle.so")
_lib = None


def build_oracle(force: bool = False) -> str:
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
        # PCMM_ORACLE_LIB names another build of the same pcmm_oracle.c (the sanitizer test compiles one
        # with -fsanitize=address,undefined and runs the pins on it)
        lib = ctypes.CDLL(os.environ.get("PCMM_ORACLE_LIB") or build_oracle())
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.pcmm_oracle_select.argtypes = [p, p, p, i64, i64, i64, i64, p, i64, p, i64, p]
        lib.pcmm_oracle_select.restype = ctypes.c_int
        lib.pcmm_oracle.argtypes = [p, p, p, i64, i64, i64, i64, p]
        lib.pcmm_oracle.restype = ctypes.c_int
        lib.pcmm_freivalds.argtypes = [p, p, p, p, ctypes.c_uint64, i64, i64, i64]
        lib.pcmm_freivalds.restype = ctypes.c_int64
        lib.pcmm_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def oracle_threads() -> int:
    """Number of host threads the oracle's OpenMP loops use."""
    return int(_load().pcmm_oracle_threads())


def _prep(W, A, primes):
    W = np.ascontiguousarray(np.asarray(W), dtype=np.int32)
    A = np.ascontiguousarray(np.asarray(A), dtype=np.uint64)
    q = np.ascontiguousarray(np.asarray([int(x) for x in primes], dtype=np.uint64))
    if W.ndim != 2 or A.ndim != 3:
        raise ValueError("W must be [M][K] and A must be [L][K][Ncols]")
    M, K = W.shape
    L, K2, Ncols = A.shape
    if K2 != K or q.shape[0] != L:
        raise ValueError("shape mismatch between W, A and the prime list")
    for j in range(L):
        if A[j].size and int(A[j].max()) >= int(q[j]):
            raise ValueError("A[%d] holds a residue that is not reduced mod q_j" % j)
    return W, A, q, M, K, Ncols, L


def pcmm_oracle(W, A, primes) -> np.ndarray:
    """C[j] = W . A[j] mod primes[j], canonical representatives; returns uint64 [L][M][Ncols]."""
    W, A, q, M, K, Ncols, L = _prep(W, A, primes)
    C = np.empty((L, M, Ncols), dtype=np.uint64)
    rc = _load().pcmm_oracle(W.ctypes.data, A.ctypes.data, q.ctypes.data, M, K, Ncols, L, C.ctypes.data)
    if rc != 0:
        raise RuntimeError("pcmm_oracle failed")
    return C


def pcmm_oracle_select(W, A, primes, rows: Sequence[int], cols: Sequence[int]) -> np.ndarray:
    """Rows `rows` and columns `cols` of every limb of C; returns uint64 [L][len(rows)][len(cols)]."""
    W, A, q, M, K, Ncols, L = _prep(W, A, primes)
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    cols = np.ascontiguousarray(np.asarray(cols, dtype=np.int64))
    C = np.empty((L, rows.size, cols.size), dtype=np.uint64)
    rc = _load().pcmm_oracle_select(
        W.ctypes.data, A.ctypes.data, q.ctypes.data, M, K, Ncols, L,
        rows.ctypes.data, rows.size, cols.ctypes.data, cols.size, C.ctypes.data,
    )
    if rc != 0:
        raise RuntimeError("pcmm_oracle_select failed (index out of range?)")
    return C


def pcmm_freivalds(W, Aj, Cj, r, q: int) -> int:
    """Number of rows of the claimed limb Cj that fail C.r = W.(A.r) mod q, plus out-of-range entries."""
    W = np.ascontiguousarray(np.asarray(W), dtype=np.int32)
    Aj = np.ascontiguousarray(np.asarray(Aj), dtype=np.uint64)
    Cj = np.ascontiguousarray(np.asarray(Cj), dtype=np.uint64)
    r = np.ascontiguousarray(np.asarray(r), dtype=np.uint64)
    M, K = W.shape
    if Aj.shape[0] != K or Cj.shape != (M, Aj.shape[1]) or r.shape != (Aj.shape[1],):
        raise ValueError("shape mismatch")
    bad = _load().pcmm_freivalds(W.ctypes.data, Aj.ctypes.data, Cj.ctypes.data, r.ctypes.data,
                                 ctypes.c_uint64(int(q)), M, K, Aj.shape[1])
    if bad < 0:
        raise RuntimeError("pcmm_freivalds: bad arguments")
    return int(bad)
