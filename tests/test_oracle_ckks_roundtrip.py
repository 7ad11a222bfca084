"""Toy CKKS encrypt -> PCMM (oracle) -> decrypt must reproduce the float64 product W.X (no GPU).

This pins that "a modular matrix product on the residues of (a | b)" is PCMM in the paper's sense:
Enc/Dec of Appendix A, component-wise Add, coefficient encoding of Section 2.1.1, B = W.A of
Section 5.1.  Each of K input rows is one ciphertext holding N real values (one channel, all
token positions); row m of the output must decrypt to sum_k W[m][k] x_k.

Error bound.  pt_k = round(Delta x_k) is off by at most 1/2 per coefficient and |e_k| <= 6 sigma,
so the decrypted integer differs from Delta * (W.X)[m][i] by at most (sum_k |W[m][k]|)(1/2 + 6 sigma);
dividing by Delta gives the bound below (plus a float64 slack of K * 2^-40).  No wrap-around
needs (sum_k |W[m][k]|)(Delta + 1/2 + 6 sigma) < Q/2, asserted.
"""
import numpy as np
import pytest

import pcmm_inputs as pi
from oracle import pcmm_oracle
from oracle import toy_ckks as ck

SIGMA = 3.2
DELTA = 1 << 30
H = 64


def _setup(N, K, primes, seed):
    rng = np.random.default_rng(seed)
    Q = 1
    for q in primes:
        Q *= int(q)
    sk_pos = rng.choice(N, size=H, replace=False)
    sk_sign = rng.choice([-1, 1], size=H)
    X = rng.uniform(-1.0, 1.0, size=(K, N))
    a_rows, b_rows = [], []
    for k in range(K):
        # uniform a in R_Q from 128 random bits per coefficient reduced mod Q (bias < 2^-50: toy)
        a = np.array([int.from_bytes(rng.bytes(16), "little") % Q for _ in range(N)], dtype=object)
        e = np.clip(np.rint(rng.normal(0.0, SIGMA, size=N)), -6 * SIGMA, 6 * SIGMA).astype(np.int64)
        ca, cb = ck.enc(ck.encode_coeff(X[k], DELTA), a, e, sk_pos, sk_sign, Q)
        a_rows.append(ca)
        b_rows.append(cb)
    return Q, sk_pos, sk_sign, X, a_rows, b_rows


@pytest.mark.parametrize(
    "N,M,K,bits,L,wmax",
    [(1 << 10, 6, 16, 36, 2, 127), (1 << 10, 4, 8, 50, 2, 4096)],
)
def test_enc_pcmm_dec_matches_float_product(N, M, K, bits, L, wmax):
    primes = pi.ntt_primes(bits, 2 * N, L)
    Q, sk_pos, sk_sign, X, a_rows, b_rows = _setup(N, K, primes, seed=2024 + bits)
    rng = np.random.default_rng(99)
    W = rng.integers(-wmax - 1, wmax + 1, size=(M, K)).astype(np.int32)

    # sanity of the toy scheme itself: decrypting an input returns its encoding up to the error
    d0 = ck.dec(a_rows[0], b_rows[0], sk_pos, sk_sign, Q)
    assert max(abs(int(v) - int(p)) for v, p in zip(d0, ck.encode_coeff(X[0], DELTA))) <= 6 * SIGMA

    # A_j[k] = [ a_k mod q_j | b_k mod q_j ]   (columns 0..N-1: a, N..2N-1: b)
    A = np.empty((L, K, 2 * N), dtype=np.uint64)
    for k in range(K):
        A[:, k, :N] = ck.to_rns(a_rows[k], primes)
        A[:, k, N:] = ck.to_rns(b_rows[k], primes)

    C = pcmm_oracle(W, A, primes)

    Y = W.astype(np.float64) @ X
    for m in range(M):
        l1 = int(np.abs(W[m].astype(np.int64)).sum())
        assert l1 * (DELTA + 0.5 + 6 * SIGMA) < Q / 2            # no wrap modulo Q
        a_out = ck.crt_lift(C[:, m, :N], primes)
        b_out = ck.crt_lift(C[:, m, N:], primes)
        dec = ck.dec(a_out, b_out, sk_pos, sk_sign, Q)
        y = np.array([int(v) for v in dec], dtype=np.float64) / float(DELTA)
        bound = l1 * (0.5 + 6 * SIGMA) / DELTA + K * 2.0 ** -40
        err = np.abs(y - Y[m]).max()
        assert err <= bound, (m, err, bound)
        # and the result is not trivially zero / the bound is not vacuous
        assert np.abs(Y[m]).max() > 100 * bound


def test_crt_lift_inverts_to_rns():
    primes = pi.ntt_primes(36, 1 << 11, 3)
    Q = primes[0] * primes[1] * primes[2]
    x = np.array([0, 1, Q - 1, Q // 2, 123456789012345678901234567 % Q], dtype=object)
    assert list(ck.crt_lift(ck.to_rns(x, primes), primes)) == list(x)


def test_negacyclic_product_wraps_with_a_sign():
    # (1 + 2X + 3X^2 + 4X^3) * X^2 = -3 - 4X + X^2 + 2X^3 in Z[X]/(X^4+1)
    a = np.array([1, 2, 3, 4], dtype=object)
    assert list(ck.negacyclic_mul_ternary(a, [2], [1])) == [-3, -4, 1, 2]
    assert list(ck.negacyclic_mul_ternary(a, [0, 3], [1, -1])) == [1 + 2, 2 + 3, 3 + 4, 4 - 1]
