"""Pins of the PCMv oracle (ring products in Z_q[X]/(X^N+1), both ciphertext components, summed over the input
ciphertexts) against hand-worked values, a library convolution, closed forms and the toy CKKS."""
import os

import numpy as np
import pytest

import pcmm_inputs as pi
from oracle import pcmv_oracle, pcmv_oracle_rows, toy_ckks

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "pcmv_example.txt")


def _golden():
    out = {}
    for line in open(GOLD):
        line = line.strip()
        if line and not line.startswith("#"):
            name, *vals = line.split()
            out[name] = [int(v) for v in vals]
    return out


def _negacyclic_by_library(p, x, q):
    """p * x mod (X^N + 1, q) from numpy's linear convolution on Python integers, folded by hand."""
    N = len(p)
    full = np.convolve(np.array([int(v) for v in p], dtype=object), np.array([int(v) for v in x], dtype=object))
    out = [int(full[n]) - (int(full[n + N]) if n + N < len(full) else 0) for n in range(N)]
    return np.array([v % q for v in out], dtype=np.uint64)


def _rand_case(rng, Mp, Kp, N, primes, wmax=1 << 15):
    pt = rng.integers(-wmax, wmax, size=(Mp, Kp, N), dtype=np.int64)
    ct = np.stack([rng.integers(0, q, size=(Kp, 2, N), dtype=np.uint64) for q in primes])
    return pt, ct


def test_hand_worked_products_with_the_wrap():
    g = _golden()
    q = g["q"][0]
    pt = np.array(g["p"], dtype=np.int64).reshape(1, 1, 4)
    ct = np.array([g["x"], g["y"]], dtype=np.uint64).reshape(1, 1, 2, 4)
    out = pcmv_oracle(pt, ct, [q])
    assert out.shape == (1, 1, 2, 4)
    assert out[0, 0, 0].tolist() == g["p_times_x"]
    assert out[0, 0, 1].tolist() == g["p_times_y"]


@pytest.mark.parametrize("Mp,Kp,N,bits,L", [(1, 1, 1, 36, 1), (2, 1, 2, 36, 2), (3, 2, 8, 36, 2), (2, 3, 16, 50, 2),
                                            (4, 1, 64, 50, 3), (2, 2, 256, 36, 2)])
def test_against_the_library_convolution(Mp, Kp, N, bits, L):
    rng = np.random.default_rng(Mp * 100 + Kp * 10 + N)
    primes = pi.ntt_primes(bits, 1 << 13, L)
    pt, ct = _rand_case(rng, Mp, Kp, N, primes)
    out = pcmv_oracle(pt, ct, primes)
    for j, q in enumerate(primes):
        for m in range(Mp):
            for c in range(2):
                want = np.zeros(N, dtype=object)
                for k in range(Kp):
                    want = (want + _negacyclic_by_library(pt[m, k], ct[j, k, c], q).astype(object)) % q
                assert (out[j, m, c] == want.astype(np.uint64)).all()
    rows = [Mp - 1, 0]
    assert (pcmv_oracle_rows(pt, ct, primes, rows) == out[:, rows]).all()


def test_monomials_shift_with_a_sign():
    """X^s * x: coefficient i moves to i + s, and picks up a minus sign when it wraps past X^N = -1."""
    rng = np.random.default_rng(1)
    N, q = 32, pi.ntt_primes(36, 1 << 13, 1)[0]
    x = rng.integers(0, q, size=N, dtype=np.uint64)
    ct = np.stack([x, x[::-1].copy()]).reshape(1, 1, 2, N)
    for s in (0, 1, 5, N - 1):
        pt = np.zeros((1, 1, N), dtype=np.int64)
        pt[0, 0, s] = -3
        out = pcmv_oracle(pt, ct, [q])[0, 0]
        for c, v in enumerate((x, x[::-1])):
            want = np.empty(N, dtype=object)
            for i in range(N):
                want[(i + s) % N] = (-3 * int(v[i]) * (1 if i + s < N else -1)) % q
            assert (out[c] == want.astype(np.uint64)).all()


def test_bilinearity_and_the_sum_over_input_ciphertexts():
    rng = np.random.default_rng(2)
    N, Kp = 32, 3
    primes = pi.ntt_primes(50, 1 << 13, 2)
    pt1, ct = _rand_case(rng, 2, Kp, N, primes)
    pt2, ct2 = _rand_case(rng, 2, Kp, N, primes)
    qs = np.array(primes, dtype=object).reshape(-1, 1, 1, 1)
    o1, o2 = pcmv_oracle(pt1, ct, primes).astype(object), pcmv_oracle(pt2, ct, primes).astype(object)
    assert (pcmv_oracle(pt1 + pt2, ct, primes).astype(object) == (o1 + o2) % qs).all()
    ct_sum = ((ct.astype(object) + ct2.astype(object)) % qs).astype(np.uint64)
    assert (pcmv_oracle(pt1, ct_sum, primes).astype(object) == (o1 + pcmv_oracle(pt1, ct2, primes).astype(object)) % qs).all()
    parts = sum(pcmv_oracle(pt1[:, k:k + 1], ct[:, k:k + 1], primes).astype(object) for k in range(Kp))
    assert (o1 == parts % qs).all()
    assert (pcmv_oracle(np.zeros_like(pt1), ct, primes) == 0).all()


def test_coefficient_zero_is_a_matrix_vector_product():
    """Coefficient encoding: with pt_r = W[r][0] - sum_{j>=1} W[r][j] X^{N-j}, the constant coefficient of pt_r * x
    is the inner product <W_r, x>: the matrix-vector meaning of the ring products (Section 3.2: PCMv)."""
    rng = np.random.default_rng(3)
    N, M = 64, 5
    primes = pi.ntt_primes(36, 1 << 13, 2)
    W = rng.integers(-(1 << 15), 1 << 15, size=(M, N), dtype=np.int64)
    x = np.stack([rng.integers(0, q, size=N, dtype=np.uint64) for q in primes])
    pt = np.zeros((M, 1, N), dtype=np.int64)
    pt[:, 0, 0] = W[:, 0]
    for j in range(1, N):
        pt[:, 0, N - j] = -W[:, j]
    ct = np.stack([x, x], axis=1).reshape(len(primes), 1, 2, N)
    out = pcmv_oracle(pt, ct, primes)
    for l, q in enumerate(primes):
        for r in range(M):
            want = sum(int(W[r, j]) * int(x[l, j]) for j in range(N)) % q
            assert int(out[l, r, 0, 0]) == want and int(out[l, r, 1, 0]) == want


def test_products_decrypt_to_the_plaintext_product_in_the_toy_ckks():
    """Dec(pt * ct) = pt * (m + e): the plaintext polynomial multiplies both components (Appendix A: Enc, Dec, PCMult)."""
    rng = np.random.default_rng(4)
    N, Kp, Mp = 64, 2, 3
    primes = pi.ntt_primes(36, 1 << 13, 2)
    Q = primes[0] * primes[1]
    sk_pos = rng.choice(N, size=16, replace=False)
    sk_sign = rng.choice([-1, 1], size=16)
    pt = rng.integers(-(1 << 10), 1 << 10, size=(Mp, Kp, N), dtype=np.int64)
    msgs, errs, cts = [], [], []
    for k in range(Kp):
        m = toy_ckks.encode_coeff(rng.uniform(-1, 1, size=N), 1 << 30)
        e = np.array([int(v) for v in np.rint(rng.normal(0, 3.2, size=N))], dtype=object)
        a = np.array([int(rng.integers(0, 1 << 62)) * int(rng.integers(0, 1 << 10)) % Q for _ in range(N)], dtype=object)
        cts.append(toy_ckks.enc(m, a, e, sk_pos, sk_sign, Q))
        msgs.append(m)
        errs.append(e)
    ct = np.empty((2, Kp, 2, N), dtype=np.uint64)
    for k, (a, b) in enumerate(cts):
        ct[:, k, 0] = toy_ckks.to_rns(a, primes)
        ct[:, k, 1] = toy_ckks.to_rns(b, primes)
    out = pcmv_oracle(pt, ct, primes)
    for r in range(Mp):
        a_out = toy_ckks.crt_lift(out[:, r, 0], primes)
        b_out = toy_ckks.crt_lift(out[:, r, 1], primes)
        got = toy_ckks.dec(a_out, b_out, sk_pos, sk_sign, Q)
        want = np.zeros(N, dtype=object)
        for k in range(Kp):
            full = np.convolve(np.array([int(v) for v in pt[r, k]], dtype=object), msgs[k] + errs[k])
            want = want + np.array([int(full[n]) - (int(full[n + N]) if n + N < len(full) else 0) for n in range(N)], dtype=object)
        assert (got == want).all()


def test_bad_arguments():
    with pytest.raises(ValueError):
        pcmv_oracle(np.zeros((1, 1, 4)), np.zeros((1, 1, 2, 8), dtype=np.uint64), [97])
    with pytest.raises(ValueError):
        pcmv_oracle(np.zeros((1, 1, 4)), np.full((1, 1, 2, 4), 97, dtype=np.uint64), [97])
    with pytest.raises(RuntimeError):
        pcmv_oracle_rows(np.zeros((1, 1, 4)), np.zeros((1, 1, 2, 4), dtype=np.uint64), [97], [1])
