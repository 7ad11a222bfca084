"""Pins of the ring-switch permutation oracle against what the paper's formula and the mathematics fix."""
import os
import random

import numpy as np
import pytest

from oracle import ring_compose, ring_decompose
from oracle import toy_ckks as tk

HERE = os.path.dirname(os.path.abspath(__file__))


def test_hand_worked_example():
    rows = {}
    with open(os.path.join(HERE, "golden", "ring_switch_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, *vals = line.split()
            rows[name] = np.array([int(v) for v in vals], dtype=np.uint64)
    parts = ring_decompose(rows["p"], 3)
    for j in range(3):
        assert (parts[j] == rows["p_%d" % j]).all()
    assert (ring_compose(parts) == rows["p"]).all()


@pytest.mark.parametrize("N,k", [(64, 1), (64, 2), (64, 8), (64, 64), (96, 3), (48, 16)])
def test_polynomial_identity_at_random_points(N, k):
    """p(x) = sum_j p_j(x^k) x^j modulo a prime, at random x, in Python integers."""
    rnd = random.Random(N * 100 + k)
    q = (1 << 61) - 1
    p = np.array([rnd.randrange(q) for _ in range(N)], dtype=object)
    parts = ring_decompose(p, k)
    assert parts.shape == (k, N // k)
    for _ in range(5):
        x = rnd.randrange(1, q)
        lhs = sum(int(c) * pow(x, i, q) for i, c in enumerate(p)) % q
        xk = pow(x, k, q)
        rhs = sum(sum(int(c) * pow(xk, i, q) for i, c in enumerate(parts[j])) * pow(x, j, q) for j in range(k)) % q
        assert lhs == rhs
    # a transposed or shifted index map breaks the identity
    if 1 < k < N:
        wrong = np.roll(parts, 1, axis=0)
        x = rnd.randrange(1, q)
        xk = pow(x, k, q)
        rhs = sum(sum(int(c) * pow(xk, i, q) for i, c in enumerate(wrong[j])) * pow(x, j, q) for j in range(k)) % q
        assert rhs != sum(int(c) * pow(x, i, q) for i, c in enumerate(p)) % q


def test_round_trip_and_degenerate_cases():
    rng = np.random.default_rng(1)
    p = rng.integers(0, 1 << 62, size=(3, 2, 128), dtype=np.uint64)
    for k in (1, 2, 4, 32, 128):
        parts = ring_decompose(p, k)
        assert parts.shape == (3, 2, k, 128 // k)
        assert (ring_compose(parts) == p).all()
    assert (ring_decompose(p, 1)[..., 0, :] == p).all()                 # k = 1: nothing moves
    assert (ring_decompose(p, 128)[..., :, 0] == p).all()               # k = N: one constant per part
    with pytest.raises(ValueError):
        ring_decompose(p, 3)


@pytest.mark.parametrize("N,k", [(256, 4), (512, 16)])
def test_parts_decrypt_under_the_subring_secret(N, k):
    """A ciphertext over R_N under the secret sk'(X^k), sk' in R_{N'}: every part (a_j, b_j) decrypts
    under sk' in R_{N'} to the coefficients j, j+k, ... of the message (Section 3.3; Appendix A for Enc/Dec)."""
    rnd = random.Random(7 * N + k)
    Np = N // k
    Q = 68719403009 * 68719230977
    h = 16
    pos_sub = sorted(rnd.sample(range(Np), h))
    sign = [rnd.choice((-1, 1)) for _ in range(h)]
    pos_big = [p * k for p in pos_sub]                                   # sk'(X^k) as an element of R_N
    pt = np.array([rnd.randrange(-(1 << 30), 1 << 30) for _ in range(N)], dtype=object)
    e = np.array([rnd.randrange(-19, 20) for _ in range(N)], dtype=object)
    a = np.array([rnd.randrange(Q) for _ in range(N)], dtype=object)
    a, b = tk.enc(pt, a, e, pos_big, sign, Q)
    assert (tk.dec(a, b, pos_big, sign, Q) == pt + e).all()
    a_parts, b_parts = ring_decompose(a, k), ring_decompose(b, k)
    want = ring_decompose(pt + e, k)
    for j in range(k):
        got = tk.dec(a_parts[j], b_parts[j], pos_sub, sign, Q)
        assert (got == want[j]).all(), j
