"""CPU oracle for the coefficient permutation of ring switching: test infrastructure only.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.

What it computes (Section 3.3, "Ring-switching in SinC encoding", the coefficient-encoding case stated
first): after the key switch to a secret of the subring R_{N'}, N' | N, k = N / N', each component p
(a' or b') of the ciphertext over R_N is decomposed as

    p(X) = sum_{j<k} p_j(X^k) X^j ,        p_j in R_{N'} ,

i.e. coefficient i of p_j is coefficient i*k + j of p.  `ring_decompose` returns the p_j,
`ring_compose` is the inverse map (sub-ring components back to one polynomial of degree N).
The key switch itself is not part of this module.  Plain numpy index arithmetic, any integer dtype
(also object arrays of Python integers).
"""
from __future__ import annotations

import numpy as np


def ring_decompose(p: np.ndarray, k: int) -> np.ndarray:
    """p[..., N] -> parts[..., k, N/k] with parts[..., j, i] = p[..., i*k + j]."""
    p = np.asarray(p)
    N = p.shape[-1]
    if k <= 0 or N % k:
        raise ValueError("k must divide the ring degree")
    parts = np.empty(p.shape[:-1] + (k, N // k), dtype=p.dtype)
    for j in range(k):
        for i in range(N // k):
            parts[..., j, i] = p[..., i * k + j]      # the coefficient of (X^k)^i X^j
    return parts


def ring_compose(parts: np.ndarray) -> np.ndarray:
    """parts[..., k, N'] -> p[..., k*N'] with p[..., i*k + j] = parts[..., j, i]."""
    parts = np.asarray(parts)
    k, Np = parts.shape[-2], parts.shape[-1]
    p = np.empty(parts.shape[:-2] + (k * Np,), dtype=parts.dtype)
    for j in range(k):
        for i in range(Np):
            p[..., i * k + j] = parts[..., j, i]
    return p
