"""Host-side model of the PCMv kernels' exact double-precision modular arithmetic, checked against Python integers.

csrc/pcmv.hip multiplies residues held as integers in doubles (mulmod), reduces them (reduce) and, at the end of the
degree-4096 transform, maps them to [0, q) (canonical); for primes below 2^36 the transform never reduces its sums, so
mulmod sees second operands up to 2^13 q and canonical sees values up to 2^12 q.  The comments there argue that every
step is exact and bound the magnitudes.  This file re-states the operations one by one (fma emulated exactly with
rationals), follows a value through the worst case the bounds allow, and checks the claims at the edges of the ranges,
so that a wrong bound shows up here, on the CPU.  It shares no code with the kernels or the oracle.
"""
import math
import random
from fractions import Fraction

import pytest

MAGIC = 6755399441055744.0     # 1.5 * 2^52


def fma(a: float, b: float, c: float) -> float:
    return float(Fraction(a) * Fraction(b) + Fraction(c))      # one rounding, like the hardware


def round_fma(h: float, s: float) -> float:
    return fma(h, s, MAGIC) - MAGIC


def mulmod(a: float, b: float, q: float, invq: float) -> float:
    h = a * b
    lo = fma(a, b, -h)
    qh = round_fma(h, invq)
    t = fma(-qh, q, h)
    assert Fraction(t) == Fraction(h) - Fraction(qh) * Fraction(q)          # the remainder step is exact
    r = t + lo
    assert Fraction(r) == Fraction(t) + Fraction(lo)                        # and so is the addition of the low part
    return r


def reduce(v: float, q: float, invq: float) -> float:
    return fma(-round_fma(v, invq), q, v)


def canonical(v: float, q: float, invq: float) -> float:
    return fma(-float(math.floor(fma(v, invq, 0.5 * invq))), q, v)


def _primes_like(bits):
    """Odd moduli at both ends of the bits-bit range (the arithmetic does not need primality)."""
    lo, hi = (1 << (bits - 1)) + 1, (1 << bits) - 1
    return [lo, lo + 2, hi, hi - 2, (lo + hi) // 2 | 1]


@pytest.mark.parametrize("bits", [24, 30, 36])
def test_lazy_multiplication_is_exact_and_small(bits):
    rng = random.Random(bits)
    for q in _primes_like(bits):
        qd, invq = float(q), 1.0 / float(q)
        amax, bmax = q // 2 + 1, (1 << 13) * q
        cases = [(amax, bmax), (-amax, bmax), (amax, -bmax), (amax, bmax - 1), (1, bmax), (amax - 1, bmax - q // 2)]
        cases += [(rng.randint(-amax, amax), rng.randint(-bmax, bmax)) for _ in range(300)]
        for a, b in cases:
            r = mulmod(float(a), float(b), qd, invq)
            assert r == int(r) and (int(r) - a * b) % q == 0
            assert abs(r) <= 0.5625 * q


@pytest.mark.parametrize("bits", [37, 44, 50])
def test_reducing_multiplication_at_its_bounds(bits):
    rng = random.Random(bits)
    for q in _primes_like(bits):
        qd, invq = float(q), 1.0 / float(q)
        amax, bmax = q // 2 + 1, 4 * q
        cases = [(amax, bmax), (-amax, bmax), (amax, -bmax), (amax, 2 * q), (amax, bmax - 1)]
        cases += [(rng.randint(-amax, amax), rng.randint(-bmax, bmax)) for _ in range(300)]
        for a, b in cases:
            r = mulmod(float(a), float(b), qd, invq)
            assert r == int(r) and (int(r) - a * b) % q == 0
            assert abs(r) <= q
            if abs(b) <= 2 * q:
                assert abs(r) <= 0.75 * q + 1


@pytest.mark.parametrize("bits", [24, 30, 36])
def test_canonical_residue_of_unreduced_values(bits):
    """|v| < 2^12 q, q < 2^36: the biased floor picks the right multiple at every edge."""
    rng = random.Random(100 + bits)
    for q in _primes_like(bits):
        qd, invq = float(q), 1.0 / float(q)
        ks = [0, 1, -1, 2, -2, 4095, -4095, -4096, 2048, -2049] + [rng.randint(-4096, 4095) for _ in range(40)]
        ss = [0, 1, 2, q - 1, q - 2, q // 2, q // 2 + 1] + [rng.randrange(q) for _ in range(10)]
        for k in ks:
            for s in ss:
                v = k * q + s
                assert abs(v) <= (1 << 12) * q
                assert canonical(float(v), qd, invq) == float(s)


def test_worst_case_growth_through_twelve_stages():
    """A sum that is never reduced doubles at most once per stage: with inputs and products bounded by 0.5625 q the
    values stay below 2^12 q < 2^48 and the differences below 2^13 q, the operand bound of the lazy multiplication."""
    q = (1 << 36) - 5
    bound = 0.5625 * q
    for _ in range(12):
        assert 2 * bound <= (1 << 13) * q          # the difference that feeds the multiplication
        bound = max(2 * bound, 0.5625 * q)         # the sum output; the product output is small again
    assert bound < (1 << 12) * q < 2 ** 48


@pytest.mark.parametrize("bits", [24, 36, 50])
def test_reduce_brings_large_sums_back(bits):
    rng = random.Random(7 + bits)
    for q in _primes_like(bits):
        qd, invq = float(q), 1.0 / float(q)
        vmax = min(4096 * q, (1 << 52) - 1) if bits <= 36 else 4 * q
        for v in [vmax, -vmax, vmax - 1, q, -q, 0, q // 2, q // 2 + 1] + [rng.randint(-vmax, vmax) for _ in range(200)]:
            r = reduce(float(v), qd, invq)
            assert r == int(r) and (int(r) - v) % q == 0 and abs(r) <= q // 2 + 1
