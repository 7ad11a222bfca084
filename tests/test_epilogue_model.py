"""Host-side model of the kernel's double-precision epilogue, checked against Python integers.

The GPU epilogue reduces sum_e acc_e 256^e modulo q with a handful of IEEE double operations whose exactness
is argued in the comments of reduce_f64 (csrc/pcmm.hip).  This file re-states those operations one by one
(fma emulated exactly with rationals) and checks the claim on the extreme accumulator patterns and primes at
the edges of every variant's range, so that a wrong bound shows up here, on the CPU, and not as a rare wrong
residue on the GPU.  It shares no code with the kernel or the oracle.
"""
import itertools
import random
from fractions import Fraction

import numpy as np
import pytest


def fma(a: float, b: float, c: float) -> float:
    return float(Fraction(a) * Fraction(b) + Fraction(c))      # one rounding, like the hardware


def rint(x: float) -> float:
    return float(np.rint(x))


def reduce_model(acc, q: int, mode: int) -> int:
    """mode 0: groups of three; 1: groups of four; 2: groups of four built from int32 pairs."""
    E = len(acc)
    gs = 3 if mode == 0 else 4
    G = (E + gs - 1) // gs
    qd, invq = float(q), 1.0 / float(q)
    c = []
    for g in range(G):
        b0 = gs * g
        if mode == 2:
            def pair(i):
                p = acc[i] + (acc[i + 1] << 8) if i + 1 < E and i + 1 < b0 + gs else acc[i]
                assert -(1 << 31) <= p < (1 << 31)                # the int32 the kernel computes in
                return p
            v = float(pair(b0))
            if b0 + 2 < E:
                v = fma(float(pair(b0 + 2)), 65536.0, v)
        else:
            v = float(acc[b0])
            for i in range(1, gs):
                if b0 + i < E:
                    v = fma(float(acc[b0 + i]), float(1 << (8 * i)), v)
        c.append(v)
    B = 16777216.0 if mode == 0 else 4294967296.0
    r = c[G - 1]
    for g in range(G - 2, -1, -1):
        X = r * B
        qh = rint((X + c[g]) * invq)
        r = fma(-qh, qd, X) + c[g]
    lift = float(np.floor(r * invq))          # -1 for a negative remainder, 0 otherwise (|r| <= 0.6 q)
    assert lift == (-1.0 if r < 0.0 else 0.0)
    r = fma(-lift, qd, r)
    assert r == int(r) and 0 <= r < 2 ** 52
    return int(r)


def exact(acc, q):
    return sum(a << (8 * e) for e, a in enumerate(acc)) % q


def odd_near(x):
    return [v for v in (x - 3, x - 1, x + 1, x + 3) if v % 2 == 1] or [x | 1]


# (mode, E values, accumulator bound, q range) as the plan selects them
VARIANTS = [
    (0, (4, 5, 6, 7, 8), (1 << 31) - 1, ((1 << 23) + 1, (1 << 50) - 1)),
    (1, (7, 8), 16383 * 16384, ((1 << 37) + 1, (1 << 50) - 1)),
    (2, (7, 8), 509 * 16384, ((1 << 37) + 1, (1 << 50) - 1)),
]


@pytest.mark.parametrize("mode,Es,amax,qrange", VARIANTS)
def test_extreme_accumulators_at_the_edges_of_the_prime_range(mode, Es, amax, qrange):
    qlo, qhi = qrange
    qs = sorted(set(odd_near(qlo + 2) + odd_near(qhi - 2) + odd_near((qlo + qhi) // 2) + odd_near(1 << 40) + odd_near(1 << 49)))
    qs = [q for q in qs if qlo <= q <= qhi]
    for E in Es:
        for signs in itertools.product((-1, 1), repeat=E):
            acc = [s * amax for s in signs]
            for q in qs:
                assert reduce_model(acc, q, mode) == exact(acc, q), (acc, q)
        # one accumulator at the bound, the others zero or the opposite bound
        for e in range(E):
            for other in (0, -amax):
                acc = [other] * E
                acc[e] = amax
                for q in qs:
                    assert reduce_model(acc, q, mode) == exact(acc, q), (acc, q)


@pytest.mark.parametrize("mode,Es,amax,qrange", VARIANTS)
def test_random_accumulators_and_primes(mode, Es, amax, qrange):
    rnd = random.Random(1234 + mode)
    qlo, qhi = qrange
    for _ in range(6000):
        E = rnd.choice(Es)
        bits = rnd.randrange(qlo.bit_length(), qhi.bit_length() + 1)
        q = rnd.randrange(max(qlo, 1 << (bits - 1)), min(qhi, (1 << bits) - 1) + 1) | 1
        q = min(q, qhi)
        scale = rnd.choice((amax, amax, amax >> 7, 300))
        acc = [rnd.randrange(-scale, scale + 1) for _ in range(E)]
        assert reduce_model(acc, q, mode) == exact(acc, q), (acc, q)


def test_values_that_are_multiples_of_q_or_one_off():
    """The residues 0 and q-1 sit at the two ends of the final lift."""
    rnd = random.Random(9)
    for mode, E, amax in ((0, 5, (1 << 27)), (1, 8, 1 << 27), (2, 8, 509 * 16384)):
        for _ in range(400):
            q = rnd.randrange((1 << 49) + 1, 1 << 50) | 1
            # build accumulators whose value is t*q + delta by peeling digits of the target
            t = rnd.randrange(-(1 << 10), 1 << 10)
            for delta in (0, 1, -1):
                target = t * q + delta
                acc, v = [], target
                for e in range(E - 1):
                    d = ((v + 128) % 256) - 128
                    acc.append(d)
                    v = (v - d) >> 8
                acc.append(v)
                if abs(acc[-1]) > amax:
                    continue
                assert sum(a << (8 * e) for e, a in enumerate(acc)) == target
                assert reduce_model(acc, q, mode) == target % q


# ---- the integer epilogues (primes of 2^50 and more): 64-bit Barrett, one piece or two pieces + Shoup
M64 = (1 << 64) - 1


def barrett_u64(u, q, mu):
    assert 0 <= u <= M64
    qhat = (u * mu) >> 64
    r = (u - qhat * q) & M64
    return r - q if r >= q else r


def mulmod_shoup(x, c, cs, q):
    qhat = (x * cs) >> 64
    r = (x * c - qhat * q) & M64
    return r - q if r >= q else r


def reduce_int_model(acc, q):
    mu = (1 << 64) // q
    off = q * ((1 << 62) // q)
    assert off >= 1 << 61
    vlo = sum(a << (8 * e) for e, a in enumerate(acc[:4]))
    vhi = sum(a << (8 * (e - 4)) for e, a in enumerate(acc) if 4 <= e < 8)
    assert abs(vlo) < 1 << 56 and abs(vhi) < 1 << 56
    c32 = (1 << 32) % q
    c32s = (c32 << 64) // q
    rlo = barrett_u64((vlo + off) & M64, q, mu)
    rhi = barrett_u64((vhi + off) & M64, q, mu)
    res = rlo + mulmod_shoup(rhi, c32, c32s, q)
    res = res - q if res >= q else res
    if len(acc) == 9:                                           # a ninth accumulator: int16 weights with 8 digits
        c64 = (1 << 64) % q
        c64s = (c64 << 64) // q
        rtop = barrett_u64((acc[8] + off) & M64, q, mu)
        res += mulmod_shoup(rtop, c64, c64s, q)
        res = res - q if res >= q else res
    return res


def test_integer_epilogues_against_python_integers():
    rnd = random.Random(77)
    amax = (1 << 31) - 1
    for bits in (50, 51, 55, 56, 61, 62):
        qs = [((1 << bits) - 1) | 1, (1 << (bits - 1)) + 1] + [rnd.randrange(1 << (bits - 1), 1 << bits) | 1 for _ in range(6)]
        for q in qs:
            for E in (7, 8, 9):
                cases = [[s * amax for s in signs] for signs in itertools.product((-1, 1), repeat=E)]
                cases += [[rnd.randrange(-amax, amax + 1) for _ in range(E)] for _ in range(300)]
                for acc in cases:
                    assert reduce_int_model(acc, q) == exact(acc, q), (acc, q)
