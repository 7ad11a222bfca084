"""Toy, INSECURE symmetric CKKS used only to pin the PCMM oracle (test infrastructure).

Follows the paper's Appendix A ("Encryption and decryption"):
  * the plaintext space is R = Z[X]/(X^N + 1); a ciphertext is a pair (a, b) in R_Q^2;
  * Enc(pt) = (a, -a*sk + pt + e mod Q) with a uniform in R_Q, e a small error, sk ternary
    with h non-zero coefficients;
  * Dec(a, b) = a*sk + b mod Q;
  * Add is component-wise, hence any integer combination sum_k w_k * ct_k decrypts to
    sum_k w_k * (pt_k + e_k): the fact the PCMM-to-clear-matrix-product reduction of
    Section 2.2 rests on.
Messages use coefficient encoding (Section 2.1.1): a real vector x becomes the polynomial
with coefficients round(Delta * x_i).

Everything is exact Python-integer arithmetic on numpy object arrays; all randomness
(a, e, sk) is passed in by the caller.  Sizes are toy sizes (N <= 2^12).
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def encode_coeff(x: np.ndarray, delta: int) -> np.ndarray:
    """Coefficient encoding of a real vector: integer polynomial round(delta * x) (object array)."""
    return np.array([int(v) for v in np.rint(np.asarray(x, dtype=np.float64) * float(delta))], dtype=object)


def negacyclic_mul_ternary(a: np.ndarray, sk_pos: Sequence[int], sk_sign: Sequence[int]) -> np.ndarray:
    """a * sk in Z[X]/(X^N+1) for sk = sum_t sign_t X^{pos_t}; exact integers, no modulus."""
    a = np.asarray(a, dtype=object)
    N = a.shape[0]
    out = np.zeros(N, dtype=object)
    for p, s in zip(sk_pos, sk_sign):
        p = int(p)
        # X^p * a(X): coefficient i moves to i+p; wrapping past N picks up a minus sign (X^N = -1)
        shifted = np.empty(N, dtype=object)
        shifted[p:] = a[: N - p]
        shifted[:p] = -a[N - p:]
        out = out + int(s) * shifted
    return out


def enc(pt: np.ndarray, a: np.ndarray, e: np.ndarray, sk_pos, sk_sign, Q: int) -> Tuple[np.ndarray, np.ndarray]:
    """(a, b) with b = -a*sk + pt + e mod Q, entries in [0, Q)."""
    a = np.asarray(a, dtype=object) % Q
    b = (-negacyclic_mul_ternary(a, sk_pos, sk_sign) + np.asarray(pt, dtype=object) + np.asarray(e, dtype=object)) % Q
    return a, b


def dec(a: np.ndarray, b: np.ndarray, sk_pos, sk_sign, Q: int) -> np.ndarray:
    """a*sk + b mod Q, centred to (-Q/2, Q/2]."""
    v = (negacyclic_mul_ternary(np.asarray(a, dtype=object), sk_pos, sk_sign) + np.asarray(b, dtype=object)) % Q
    return np.array([int(x) - Q if int(x) > Q // 2 else int(x) for x in v], dtype=object)


def to_rns(x: np.ndarray, primes: Sequence[int]) -> np.ndarray:
    """Residues of an integer vector modulo each prime: uint64 [L][len(x)]."""
    x = np.asarray(x, dtype=object)
    return np.stack([np.array([int(v) % int(q) for v in x], dtype=np.uint64) for q in primes])


def crt_lift(res: np.ndarray, primes: Sequence[int]) -> np.ndarray:
    """Inverse of to_rns: the unique integers in [0, Q) with the given residues (object array)."""
    primes = [int(q) for q in primes]
    Q = 1
    for q in primes:
        Q *= q
    out = np.zeros(res.shape[1], dtype=object)
    for j, q in enumerate(primes):
        Qj = Q // q
        coef = Qj * pow(Qj, -1, q)
        out = out + np.array([int(v) for v in res[j]], dtype=object) * coef
    return out % Q
