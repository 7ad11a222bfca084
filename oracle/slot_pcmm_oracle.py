"""CPU oracle for the slot-encoded batch PCMM of PC-attention (Section 4.2; correctness in Appendix E).

TEST INFRASTRUCTURE ONLY: nothing in the product path may import this file.  It shares no code with
the HIP library.

What the paper fixes.  Matrices are d x d and are stored in the slots row after row.  Four index
maps are defined (all indices modulo d):

    rot_C^k(A)[i][j] = A[i][j+k]        sigma(A)[i][j] = A[i][i+j]
    rot_R^k(A)[i][j] = A[i+k][j]        tau(A)[i][j]   = A[i+j][j]

The matrix product is a sum of d Hadamard products (Eq. "JKLS"):
    C = sum_k rot_C^k(sigma(A)) (.) rot_R^k(tau(B)),
Theorem 1 (Appendix E) moves tau^l through it, and Eq. "pcmm" regroups the d terms as g giant steps of
b baby steps (g b = d):
    tau^l(C) = sum_{j<g} rot_R^{j b}( sum_{i<b} pt_{A,i,j,l} (.) rot_R^i(tau^{l+1}(B)) ),
    pt_{A,i,j,l} = rot_R^{-l (i+j b) - j b} o rot_C^{i+j b}( tau^l o sigma(A) ).
Only tau^l o sigma(A) is stored; every pt_{A,i,j,l} is made from it at run time by the two rotations.

Everything here is the definition written out with explicit loops over (i, j) on exact Python/NumPy
integers: no closed forms, no vectorised index tricks.  On clear matrices the Hadamard products act on
the entries themselves, which is what these identities are about; the homomorphic evaluation (rotations
of ciphertexts, key switching) is not part of this oracle.

Parity status: pinned by tests/test_slot_pcmm_oracle.py (hand-worked 3 x 3 example, Eq. "JKLS" against
the plain matrix product, Lemma 2, Theorem 1 and Eq. "pcmm" against tau^l of the plain product for
every factorisation g b = d, planted-mistake checks).
"""
from __future__ import annotations

import numpy as np


def _square(A) -> int:
    A = np.asarray(A)
    if A.ndim != 2 or A.shape[0] != A.shape[1]:
        raise ValueError("square matrices only")
    return A.shape[0]


def rot_col(A, k: int):
    """rot_C^k(A)[i][j] = A[i][(j + k) mod d]  (Section 4.2)."""
    d = _square(A)
    out = np.empty_like(np.asarray(A))
    for i in range(d):
        for j in range(d):
            out[i][j] = A[i][(j + k) % d]
    return out


def rot_row(A, k: int):
    """rot_R^k(A)[i][j] = A[(i + k) mod d][j]  (Section 4.2)."""
    d = _square(A)
    out = np.empty_like(np.asarray(A))
    for i in range(d):
        for j in range(d):
            out[i][j] = A[(i + k) % d][j]
    return out


def sigma(A):
    """sigma(A)[i][j] = A[i][(i + j) mod d]  (Section 4.2)."""
    d = _square(A)
    out = np.empty_like(np.asarray(A))
    for i in range(d):
        for j in range(d):
            out[i][j] = A[i][(i + j) % d]
    return out


def tau(A):
    """tau(A)[i][j] = A[(i + j) mod d][j]  (Section 4.2)."""
    d = _square(A)
    out = np.empty_like(np.asarray(A))
    for i in range(d):
        for j in range(d):
            out[i][j] = A[(i + j) % d][j]
    return out


def tau_inverse(A):
    """The map that undoes tau: out[(i + j) mod d][j] = A[i][j]."""
    d = _square(A)
    out = np.empty_like(np.asarray(A))
    for i in range(d):
        for j in range(d):
            out[(i + j) % d][j] = A[i][j]
    return out


def tau_pow(A, ell: int):
    """tau applied ell times (its inverse -ell times for negative ell)."""
    out = np.array(A, copy=True)
    for _ in range(abs(ell)):
        out = tau(out) if ell > 0 else tau_inverse(out)
    return out


def jkls_product(A, B):
    """Eq. "JKLS": sum_k rot_C^k(sigma(A)) (.) rot_R^k(tau(B))."""
    d = _square(A)
    sA, tB = sigma(A), tau(B)
    acc = np.zeros_like(np.asarray(A))
    for k in range(d):
        acc = acc + rot_col(sA, k) * rot_row(tB, k)
    return acc


def theorem1(A, B, ell: int):
    """Theorem 1 (Appendix E): sum_k (rot_R^{-ell k} o rot_C^k(tau^ell o sigma(A))) (.) rot_R^k(tau^{ell+1}(B))."""
    d = _square(A)
    S = tau_pow(sigma(A), ell)
    T = tau_pow(B, ell + 1)
    acc = np.zeros_like(np.asarray(A))
    for k in range(d):
        acc = acc + rot_row(rot_col(S, k), -ell * k) * rot_row(T, k)
    return acc


def stored_plaintext(A, ell: int):
    """tau^ell o sigma(pt_A): the one rearrangement of the plaintext matrix that is kept in memory (Section 4.2)."""
    return tau_pow(sigma(A), ell)


def rearranged_plaintext(S, i: int, j: int, ell: int, b: int):
    """pt_{A,i,j,ell} = rot_R^{-ell (i + j b) - j b} o rot_C^{i + j b}(S) with S = tau^ell o sigma(pt_A) (Section 4.2)."""
    k = i + j * b
    return rot_row(rot_col(S, k), -ell * k - j * b)


def rearranged_plaintexts(S, ell: int, g: int, b: int):
    """All g b rearranged plaintexts, indexed [j][i] (giant step, baby step)."""
    d = _square(S)
    if g * b != d:
        raise ValueError("g b must equal d")
    return np.stack([np.stack([rearranged_plaintext(S, i, j, ell, b) for i in range(b)]) for j in range(g)])


def pcmm_bsgs(A, B_tau, ell: int, g: int, b: int):
    """Eq. "pcmm": tau^ell(A B) from pt_A = A and B_tau = tau^{ell+1}(B), g giant steps of b baby steps."""
    d = _square(A)
    if g * b != d:
        raise ValueError("g b must equal d")
    S = stored_plaintext(A, ell)
    acc = np.zeros_like(np.asarray(A))
    for j in range(g):
        inner = np.zeros_like(np.asarray(A))
        for i in range(b):
            inner = inner + rearranged_plaintext(S, i, j, ell, b) * rot_row(B_tau, i)
        acc = acc + rot_row(inner, j * b)
    return acc
